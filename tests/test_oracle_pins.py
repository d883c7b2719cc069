"""Pins of the CPU oracle against things other than itself: hand-worked values, exact rational
arithmetic, closed forms, library routines on special cases, invariants, brute force, and the
published Philox known-answer vectors.  CPU only."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import PER_COL, PER_ROW, PER_TENSOR

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
QMAX = {2: 1, 3: 3, 4: 7, 5: 15, 6: 31, 7: 63, 8: 127}


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


# ------------------------------------------------------------------------------ absmax (Sec 3.1)
def test_absmax_matches_library_max_all_granularities():
    x = rng(1).standard_normal((37, 53)).astype(np.float32)
    assert oracle.absmax(x)[0] == np.abs(x).max()
    np.testing.assert_array_equal(oracle.absmax(x, PER_ROW), np.abs(x).max(axis=1))
    np.testing.assert_array_equal(oracle.absmax(x, PER_COL), np.abs(x).max(axis=0))
    assert oracle.absmax(x, PER_ROW).shape == (37,) and oracle.absmax(x, PER_COL).shape == (53,)


def test_absmax_is_max_of_magnitude_not_of_value():
    # Sec. 3.1 writes max(x) but Eq. 2 and Eq. 5 write max|x|: the most negative entry must win
    x = np.array([[0.5, -3.0, 2.0]], dtype=np.float32)
    assert oracle.absmax(x)[0] == np.float32(3.0)


def test_absmax_invariances_and_running_max():
    r = rng(2)
    x = r.standard_normal((16, 16)).astype(np.float32)
    assert oracle.absmax(-x)[0] == oracle.absmax(x)[0]
    assert oracle.absmax(r.permutation(x.ravel()).reshape(16, 16))[0] == oracle.absmax(x)[0]
    x2 = (3 * r.standard_normal((16, 16))).astype(np.float32)
    run = oracle.absmax(x2, PER_ROW, running=oracle.absmax(x, PER_ROW))
    np.testing.assert_array_equal(run, np.maximum(np.abs(x).max(1), np.abs(x2).max(1)))
    assert oracle.absmax(np.zeros((3, 3), np.float32))[0] == 0.0


# ------------------------------------------------------------------- per-bit constants (Eq. 1)
def test_qmax_table_and_constants_are_single_fp32_divisions():
    for b, q in QMAX.items():
        assert oracle.qmax(b) == q == 2 ** (b - 1) - 1
        for m in (1.0, 0.2, 3.7519, 1e-3, 117.25):
            s, inv = oracle.bit_constants(m, b)
            assert s == np.float32(m) / np.float32(q)
            assert inv == np.float32(q) / np.float32(m)
        assert oracle.bit_constants(0.0, b) == (0.0, 0.0)
    np.testing.assert_array_equal(oracle.scale_from_absmax([2.0, 0.0, 7.0], 4),
                                  np.array([2.0, 0.0, 7.0], np.float32) / np.float32(7))


# --------------------------------------------------------------------------- codes (Eq. 1)
def _golden_hand_example():
    rows = []
    with open(os.path.join(GOLDEN, "quantizer_hand_example.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            b, codes, terms = [p.strip() for p in line.split("|")]
            sse = sum(Fraction(t) for t in terms.split())
            rows.append((int(b), [int(c) for c in codes.split()], sse))
    return rows


def test_hand_worked_example_codes_and_sse():
    x = np.array([[-1, -0.5, 0, 0.26, 1]], dtype=np.float32)
    m = oracle.absmax(x)
    assert m[0] == 1.0
    for b, codes, sse in _golden_hand_example():
        y, c, _ = oracle.fake_quant(x, m, b)
        assert c.ravel().tolist() == codes
        np.testing.assert_allclose(y.ravel(), np.array(codes) / QMAX[b], rtol=1e-7)
        got = oracle.quant_error(x, m, b, b)[0, 0]
        assert got == pytest.approx(float(sse), rel=2e-5)  # fp32(0.26) vs decimal 0.26


def test_ties_round_half_to_even():
    for b, q in QMAX.items():
        # absmax = qmax makes inv = scale = 1 exactly, so codes are RNE of x itself
        x = np.array([[0.5, -0.5, 1.5, -1.5, 2.5, -2.5, 0.49999997, 0.50000006]], np.float32)
        _, c, _ = oracle.fake_quant(x, [float(q)], b)
        expect = np.clip(np.array([0, 0, 2, -2, 2, -2, 0, 1]), -q, q)
        assert c.ravel().tolist() == expect.tolist()


def test_codes_equal_exact_rational_eq1():
    """Eq. 1 evaluated in exact rational arithmetic with alpha = 1/m exact (m = qmax * 2^k makes
    qmax/m a power of two): code = RNE(clip(x/m) * qmax)."""
    r = rng(3)
    for b, q in QMAX.items():
        for k in (-3, 0, 2):
            m = float(q) * 2.0 ** k
            x = (r.standard_normal(400) * m * 0.6).astype(np.float32)
            x[:4] = [m, -m, 1.7 * m, -2.5 * m]  # on and beyond the clipping range
            _, c, _ = oracle.fake_quant(x.reshape(1, -1), [m], b)
            for xv, cv in zip(x.tolist(), c.ravel().tolist()):
                u = Fraction(xv) / Fraction(m)
                u = max(Fraction(-1), min(Fraction(1), u)) * q
                fl = math.floor(u)
                frac = u - fl
                rne = fl + (1 if frac > Fraction(1, 2) or (frac == Fraction(1, 2) and fl % 2) else 0)
                assert cv == rne


def test_codes_use_exact_product_with_fp32_reciprocal():
    """General absmax: code = RNE of the exact real product x * fl32(qmax/m), checked with
    rationals; and the magic-number fused path (fma(x, inv, 1.5*2^23) - 1.5*2^23) gives the same."""
    r = rng(4)
    x = r.standard_normal(3000).astype(np.float32)
    m = float(np.abs(x).max())
    for b, q in QMAX.items():
        _, inv = oracle.bit_constants(m, b)
        _, c, _ = oracle.fake_quant(x.reshape(1, -1), [m], b)
        for xv, cv in zip(x.tolist(), c.ravel().tolist()):
            u = Fraction(xv) * Fraction(float(inv))
            fl = math.floor(u)
            frac = u - fl
            rne = fl + (1 if frac > Fraction(1, 2) or (frac == Fraction(1, 2) and fl % 2) else 0)
            assert cv == max(-q, min(q, rne))
    # fused magic-number path on a large sample, emulated in double (x*inv exact, the sum is
    # rounded once to fp32 by the cast; double rounding can only matter within 2^-29 of a tie)
    xs = r.standard_normal(2_000_000).astype(np.float32)
    ms = float(np.abs(xs).max())
    for b in (4, 8):
        _, inv = oracle.bit_constants(ms, b)
        t = (xs.astype(np.float64) * np.float64(inv) + 12582912.0).astype(np.float32)
        magic = (t - np.float32(12582912.0)).astype(np.int32)
        _, c, _ = oracle.fake_quant(xs.reshape(1, -1), [ms], b)
        np.testing.assert_array_equal(c.ravel().astype(np.int32), magic)


def test_codes_range_symmetry_scaling_idempotence_clamp():
    r = rng(5)
    x = r.standard_normal((24, 40)).astype(np.float32)
    m = oracle.absmax(x)
    for b, q in QMAX.items():
        y, c, _ = oracle.fake_quant(x, m, b)
        assert c.min() >= -q and c.max() <= q and abs(c).max() == q
        _, cneg, _ = oracle.fake_quant(-x, m, b)
        np.testing.assert_array_equal(cneg, -c)
        _, c8, _ = oracle.fake_quant(x * np.float32(8), m * np.float32(8), b)
        np.testing.assert_array_equal(c8, c)
        y2, c2, _ = oracle.fake_quant(y, m, b)  # same absmax argument
        np.testing.assert_array_equal(c2, c)
        np.testing.assert_array_equal(y2, y)
        # absmax smaller than the data: codes saturate at +-qmax, never beyond
        _, cs, _ = oracle.fake_quant(x, m * np.float32(0.25), b)
        assert cs.min() == -q and cs.max() == q
    yz, cz, _ = oracle.fake_quant(np.zeros((2, 4), np.float32), [0.0], 4)
    assert not yz.any() and not cz.any()


def test_per_channel_codes_use_the_right_axis():
    r = rng(6)
    x = r.standard_normal((5, 8)).astype(np.float32) * np.arange(1, 6, dtype=np.float32)[:, None]
    for gran, axis in ((PER_ROW, 1), (PER_COL, 0)):
        m = oracle.absmax(x, gran)
        y, c, _ = oracle.fake_quant(x, m, 5, gran)
        # each channel, quantized alone as its own tensor, must give the same codes
        for ch in range(m.size):
            sl = x[ch:ch + 1, :] if axis == 1 else x[:, ch:ch + 1]
            _, cc, _ = oracle.fake_quant(np.ascontiguousarray(sl), m[ch:ch + 1], 5)
            got = c[ch:ch + 1, :] if axis == 1 else c[:, ch:ch + 1]
            np.testing.assert_array_equal(got, cc)


def test_half_step_error_bound():
    r = rng(7)
    x = r.standard_normal((64, 64)).astype(np.float32)
    m = oracle.absmax(x)
    for b, q in QMAX.items():
        s, _ = oracle.bit_constants(float(m[0]), b)
        y, _, _ = oracle.fake_quant(x, m, b)
        err = np.abs(y.astype(np.float64) - x.astype(np.float64))
        assert err.max() <= float(s) / 2 * (1 + q * 2.0 ** -21)
        assert err.max() > 0.4 * float(s)  # the bound is approached, not vacuous


# ------------------------------------------------------------------------ SSE / E_QE (Eq. 2)
def test_sse_brute_force_closed_form_and_invariances():
    r = rng(8)
    x = r.uniform(-1, 1, (300, 400)).astype(np.float32)
    m = oracle.absmax(x)
    sse = oracle.quant_error(x, m)
    assert sse.shape == (1, 7)
    for i, b in enumerate(range(2, 9)):
        y, c, _ = oracle.fake_quant(x, m, b)
        s_b, _ = oracle.bit_constants(float(m[0]), b)
        grid = c.astype(np.float64) * np.float64(s_b)       # the grid point, exactly
        brute = math.fsum(((grid - x.astype(np.float64)) ** 2).ravel().tolist())
        assert sse[0, i] == pytest.approx(brute, rel=1e-12)
        # the fp32 dequantized tensor is that grid point rounded once: same sum to ~1e-5
        viay = math.fsum(((y.astype(np.float64) - x.astype(np.float64)) ** 2).ravel().tolist())
        assert sse[0, i] == pytest.approx(viay, rel=1e-4)
    # dense uniform data on a fine grid: mean squared rounding error -> step^2 / 12
    s8, _ = oracle.bit_constants(float(m[0]), 8)
    assert sse[0, 6] / x.size == pytest.approx(float(s8) ** 2 / 12, rel=0.02)
    # exact scalings and symmetries
    np.testing.assert_array_equal(oracle.quant_error(x * np.float32(4), m * np.float32(4)), 16 * sse)
    np.testing.assert_array_equal(oracle.quant_error(-x, m), sse)
    perm = r.permutation(x.ravel()).reshape(x.shape)
    np.testing.assert_allclose(oracle.quant_error(perm, m), sse, rtol=1e-11)
    # sub-range of bit-widths is the matching slice
    np.testing.assert_array_equal(oracle.quant_error(x, m, 3, 5), sse[:, 1:4])
    # falls roughly 4x per bit on smooth data (9x from 2 to 3 bits: (3/1)^2)
    assert 3.0 < sse[0, 4] / sse[0, 5] < 5.0 and 6.0 < sse[0, 0] / sse[0, 1] < 12.0



def test_two_bit_error_is_the_distance_to_the_nearest_of_minus_m_zero_m():
    """For b = 2 the grid of Eq. 1 is {-m, 0, +m} (qmax = 1, step = m): the error of an element is
    its distance to the nearest of the three points, min(|x|, ||x| - m|), also for |x| > m (the clip)
    and for m = 0.  Independent of the rounding recipe, so it pins the two-bit column of Eq. 2's sum;
    the library's sweep kernels use exactly this form for two bits."""
    r = rng(37)
    for shape, m_scale in (((53, 67), 1.0), ((40, 33), 0.5), ((9, 11), 0.0)):
        x = r.standard_normal(shape).astype(np.float32)
        x.ravel()[:5] = [0.0, 1.0, -1.0, 0.5, -0.5]
        m = (oracle.absmax(x) * np.float32(m_scale)).astype(np.float32)   # own maximum, a foreign smaller one, zero
        mm = float(m[0])
        x.ravel()[5:8] = [mm / 2, -mm / 2, mm]                             # the midpoints (ties) and the grid point itself
        a = np.abs(x.astype(np.float64))
        want = math.fsum((np.minimum(a, np.abs(a - mm)) ** 2).ravel().tolist())
        got = oracle.quant_error(x, m, 2, 2)[0, 0]
        assert abs(got - want) <= 1e-12 * max(want, 1e-300)
        # per row, with each row's own maximum
        mr = oracle.absmax(x, oracle.PER_ROW)
        want_r = [math.fsum((np.minimum(np.abs(row.astype(np.float64)), np.abs(np.abs(row.astype(np.float64)) - float(k))) ** 2).tolist())
                  for row, k in zip(x, mr)]
        np.testing.assert_allclose(oracle.quant_error(x, mr, 2, 2, oracle.PER_ROW)[:, 0], want_r, rtol=1e-12, atol=0)


def test_sse_of_a_tensor_lying_on_the_grid():
    """Eq. 2 is stated over the reals: Q_b(x) inside the sum is the grid point code * scale_b itself.
    A tensor whose every element is such a grid point therefore has SSE_b == 0 exactly.  With a
    power-of-two step (m = qmax_b * 2^-k) every grid point is an fp32 number, so the case can be
    built without rounding; the other bit-widths of the same sweep see an off-grid tensor."""
    r = rng(31)
    for b in range(2, 9):
        q = QMAX[b]
        step = np.float32(2.0 ** -5)
        codes = r.integers(-q, q + 1, size=(37, 53))
        codes[0, 0], codes[0, 1] = q, -q                      # the absmax is attained
        x = (codes * step).astype(np.float32)                 # exact products
        m = oracle.absmax(x)
        assert float(m[0]) == q * float(step)
        s_b, inv_b = oracle.bit_constants(float(m[0]), b)
        assert float(s_b) == float(step) and float(inv_b) == 1.0 / float(step)
        _, c, _ = oracle.fake_quant(x, m, b)
        np.testing.assert_array_equal(c, codes)
        sse = oracle.quant_error(x, m)[0]
        assert sse[b - 2] == 0.0
        if b < 8 and b > 2:
            assert sse[b - 3] > 0.0                            # a coarser grid does not contain it
    # a step with a full mantissa: x = fl32(code * step) is the grid point rounded once, so the
    # sum is the sum of the squared rounding errors of those products -- tiny, not zero
    m = np.array([0.7321], np.float32)
    s8, _ = oracle.bit_constants(float(m[0]), 8)
    codes = r.integers(-127, 128, size=(64, 64))
    x = (codes.astype(np.float32) * s8).astype(np.float32)
    want = math.fsum(((codes.astype(np.float64) * np.float64(s8) - x.astype(np.float64)) ** 2).ravel().tolist())
    got = oracle.quant_error(x, m, 8, 8)[0, 0]
    assert 0.0 < want < (2.0 ** -24 * 0.7321) ** 2 * x.size
    assert got == pytest.approx(want, rel=1e-12)


def test_per_channel_sse_adds_up_and_uses_the_right_axis():
    r = rng(9)
    x = r.standard_normal((12, 20)).astype(np.float32)
    m = oracle.absmax(x)
    total = oracle.quant_error(x, m)
    rows = oracle.quant_error(x, np.full(12, m[0], np.float32), gran=PER_ROW)
    cols = oracle.quant_error(x, np.full(20, m[0], np.float32), gran=PER_COL)
    assert rows.shape == (12, 7) and cols.shape == (20, 7)
    np.testing.assert_allclose(rows.sum(0), total[0], rtol=1e-12)
    np.testing.assert_allclose(cols.sum(0), total[0], rtol=1e-12)
    # a channel swept alone equals its row of the per-channel result
    mr = oracle.absmax(x, PER_ROW)
    pr = oracle.quant_error(x, mr, gran=PER_ROW)
    np.testing.assert_allclose(oracle.quant_error(x[3:4], mr[3:4])[0], pr[3], rtol=1e-13)
    mc = oracle.absmax(x, PER_COL)
    pc = oracle.quant_error(x, mc, gran=PER_COL)
    np.testing.assert_allclose(oracle.quant_error(np.ascontiguousarray(x[:, 7:8]), mc[7:8])[0], pc[7],
                               rtol=1e-13)


def test_eqe_is_normalised_rmse_and_matches_textbook_int8():
    r = rng(10)
    x = r.standard_normal((128, 128)).astype(np.float32)
    m = oracle.absmax(x)
    sse = oracle.quant_error(x, m)[0]
    e8 = oracle.eqe(sse[6], x.size, float(m[0]))
    # textbook symmetric absmax int8 quantization with numpy (division form)
    xd = x.astype(np.float64)
    step = float(m[0]) / 127.0
    ref = np.sqrt(np.mean((np.clip(np.rint(xd / step), -127, 127) * step - xd) ** 2)) / float(m[0])
    assert e8 == pytest.approx(ref, rel=1e-4)
    # invariant to power-of-two rescaling and to sign, as Eq. 2 is
    sse2 = oracle.quant_error(x * np.float32(-0.5), m * np.float32(0.5))[0]
    assert oracle.eqe(sse2[6], x.size, float(m[0]) * 0.5) == pytest.approx(e8, rel=1e-14)
    assert oracle.eqe(0.0, 10, 0.0) == 0.0


def test_eqe_with_one_scale_per_channel():
    """Eq. 2 when every output channel has its own scale: the root of the mean squared error over ALL
    elements, relative to the tensor's max|x| -- against numpy on the dequantized tensor, and reducing
    to the per-tensor value when all channels are given the tensor's maximum."""
    r = rng(12)
    x = (r.standard_normal((24, 96)) * np.linspace(0.1, 3.0, 24)[:, None]).astype(np.float32)
    mr = oracle.absmax(x, PER_ROW)
    got = oracle.eqe_channels(oracle.quant_error(x, mr, gran=PER_ROW), x.size, mr)
    for i, b in enumerate(range(2, 9)):
        y, _, _ = oracle.fake_quant(x, mr, b, PER_ROW)
        rmse = np.sqrt(np.mean((y.astype(np.float64) - x.astype(np.float64)) ** 2))
        assert got[i] == pytest.approx(rmse / float(np.abs(x).max()), rel=1e-5)
    mt = oracle.absmax(x)
    same = np.full(24, mt[0], np.float32)
    per_t = oracle.quant_error(x, mt)[0]
    np.testing.assert_allclose(oracle.eqe_channels(oracle.quant_error(x, same, gran=PER_ROW), x.size, same),
                               [oracle.eqe(s, x.size, float(mt[0])) for s in per_t], rtol=1e-12)
    # finer scales can only help: per-channel E_QE <= per-tensor E_QE here (rows differ 30-fold in range)
    assert np.all(got < [oracle.eqe(s, x.size, float(mt[0])) for s in per_t])
    assert np.all(oracle.eqe_channels(np.zeros((3, 7)), 12, np.zeros(3, np.float32)) == 0.0)


# ------------------------------------------------------------------- noise (Eq. 3-5) and its RNG
def test_philox_published_known_answers():
    n = 0
    with open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            v = [int(t, 16) for t in line.split()]
            assert oracle.philox4x32_10(v[0:4], v[4:6]) == v[6:10]
            n += 1
    assert n == 3


def test_log_and_sincos_recipes_against_libm():
    r = rng(11)
    ks = np.concatenate([[1, 2, 3, 2 ** 24, 2 ** 24 - 1, 2 ** 23, 11863283, 11863284],
                         r.integers(1, 2 ** 24 + 1, 4000)])
    for k in ks.tolist():
        want = -2.0 * math.log(k * 2.0 ** -24)
        got = float(oracle.neg2log_u24(k))
        assert got >= 0.0
        assert abs(got - want) <= 4e-7 * max(1.0, want)
    assert float(oracle.neg2log_u24(2 ** 24)) == 0.0
    js = np.concatenate([[0, 1, 2 ** 21 - 1, 2 ** 21, 2 ** 22, 2 ** 23, 3 * 2 ** 22, 2 ** 24 - 1],
                         r.integers(0, 2 ** 24, 4000)])
    for j in js.tolist():
        c, s = oracle.sincos_2pi_u24(j)
        a = 2 * math.pi * j * 2.0 ** -24
        assert abs(float(c) - math.cos(a)) < 1.5e-7 and abs(float(s) - math.sin(a)) < 1.5e-7
    assert oracle.sincos_2pi_u24(0) == (1.0, 0.0)
    assert oracle.sincos_2pi_u24(2 ** 22) == (0.0, 1.0)


def test_gauss4_is_box_muller_of_the_philox_words():
    for g in (0, 1, 12345, 2 ** 33 + 5):
        seed, sid = 0x0123456789ABCDEF, 0xFEDCBA9876543210
        w = oracle.philox4x32_10([g & 0xFFFFFFFF, g >> 32, sid & 0xFFFFFFFF, sid >> 32],
                                 [seed & 0xFFFFFFFF, seed >> 32])
        z = oracle.gauss4(seed, sid, g)
        for p in range(2):
            u1 = ((w[2 * p] >> 8) + 1) * 2.0 ** -24
            u2 = (w[2 * p + 1] >> 8) * 2.0 ** -24
            rad = math.sqrt(-2 * math.log(u1))
            assert float(z[2 * p]) == pytest.approx(rad * math.cos(2 * math.pi * u2), abs=3e-6)
            assert float(z[2 * p + 1]) == pytest.approx(rad * math.sin(2 * math.pi * u2), abs=3e-6)


def test_noise_distribution_determinism_and_linearity():
    from scipy import stats
    n = 1 << 20
    zero = np.zeros((1024, n // 1024), np.float32)
    am = np.array([7.0], np.float32)  # b = 4: scale = 1 exactly, so y = z when lambda = 1, x = 0
    z = oracle.noise_inject(zero, am, 4, 1.0, seed=42, stream_id=7)
    assert abs(z.mean()) < 4 / math.sqrt(n)
    assert abs(z.var() - 1) < 4 * math.sqrt(2 / n)
    assert np.abs(z).max() <= math.sqrt(2 * 24 * math.log(2)) + 1e-5
    assert stats.kstest(z.ravel()[:200_000].astype(np.float64), "norm").pvalue > 1e-3
    assert abs(stats.skew(z.ravel())) < 0.02 and abs(stats.kurtosis(z.ravel())) < 0.04
    # element i depends on (seed, stream, i) only: shape, sub-ranges and b do not matter
    z2 = oracle.noise_inject(zero.reshape(256, -1), am, 4, 1.0, 42, 7)
    np.testing.assert_array_equal(z2.ravel(), z.ravel())
    z8 = oracle.noise_inject(zero[:4], np.array([127.0], np.float32), 8, 1.0, 42, 7)
    np.testing.assert_array_equal(z8, z[:4])
    assert not np.array_equal(oracle.noise_inject(zero[:4], am, 4, 1.0, 43, 7), z[:4])
    assert not np.array_equal(oracle.noise_inject(zero[:4], am, 4, 1.0, 42, 8), z[:4])
    # element i takes lane (i mod 4) of group (i div 4); gauss4 itself is pinned above
    for i in (0, 1, 2, 3, 4, 1023, 1024, 4097, n - 1):
        assert z.ravel()[i] == oracle.gauss4(42, 7, i >> 2)[i & 3]
    # lambda = 0 leaves x alone; power-of-two lambda scales the perturbation exactly
    x = rng(12).standard_normal((4, 1024)).astype(np.float32)
    np.testing.assert_array_equal(oracle.noise_inject(x, am, 4, 0.0, 42, 7), x)
    np.testing.assert_array_equal(oracle.noise_inject(zero[:4], am, 4, 0.25, 42, 7), z[:4] * np.float32(0.25))
    # y = fl32(x + sigma z), one rounding: compare with the double sum rounded once
    y = oracle.noise_inject(x, am, 4, 0.5, 42, 7)
    want = (x.astype(np.float64) + 0.5 * z[:4].astype(np.float64)).astype(np.float32)
    np.testing.assert_array_equal(y, want)
    # per-row spread follows each row's absmax
    amr = np.array([7.0, 14.0, 0.0, 3.5], np.float32)
    yr = oracle.noise_inject(zero[:4], amr, 4, 1.0, 42, 7, gran=PER_ROW)
    np.testing.assert_array_equal(yr, z[:4] * np.array([1, 2, 0, 0.5], np.float32)[:, None])


# --------------------------------------------------------------------------- qgemm and packing
def test_qgemm_hand_example_and_epilogue_order():
    a = np.array([[1, -2], [3, 4]], np.int8)
    w = np.array([[5, 6], [-7, 8]], np.int8)
    y, acc = oracle.qgemm(a, w, [0.5], [0.25, 2.0], w_gran=PER_ROW)
    assert acc.tolist() == [[-7, -23], [39, 11]]
    assert y.tolist() == [[-0.875, -23.0], [4.875, 11.0]]
    # (float(acc) * s_A) * s_W, in that order, each product rounded to fp32
    acc1 = 30_000_001
    a1 = np.full((1, 1861), 127, np.int8)
    w1 = np.full((1, 1861), 127, np.int8)  # 1861 * 16129 = 30_016_069
    sa, sw = np.float32(0.1234567), np.float32(7.654321)
    y1, c1 = oracle.qgemm(a1, w1, [sa], [sw])
    assert int(c1[0, 0]) == 1861 * 16129
    assert y1[0, 0] == np.float32(np.float32(np.float32(1861 * 16129) * sa) * sw)


def test_qgemm_brute_force_against_wide_integer_matmul():
    r = rng(13)
    for (M, N, K) in [(1, 1, 2), (3, 5, 7), (17, 9, 64), (33, 31, 130), (2, 3, 4608)]:
        a = r.integers(-127, 128, (M, K)).astype(np.int8)
        w = r.integers(-127, 128, (N, K)).astype(np.int8)
        _, acc = oracle.qgemm(a, w, [1.0], [1.0])
        np.testing.assert_array_equal(acc, a.astype(np.int64) @ w.astype(np.int64).T)
    a = r.integers(-127, 128, (6, 6)).astype(np.int8)
    _, acc = oracle.qgemm(a, np.eye(6, dtype=np.int8), [1.0], [1.0])
    np.testing.assert_array_equal(acc, a)
    _, acc = oracle.qgemm(a, np.ones((2, 6), np.int8), [1.0], [1.0])
    np.testing.assert_array_equal(acc, np.repeat(a.astype(np.int32).sum(1, keepdims=True), 2, 1))
    # extreme operands at the largest configured K stay inside int32; far larger K is reported
    big = np.full((1, 4608), -127, np.int8)
    _, acc = oracle.qgemm(big, -big, [1.0], [1.0])
    assert int(acc[0, 0]) == -4608 * 127 * 127
    huge = np.full((1, 133200), 127, np.int8)
    with pytest.raises(RuntimeError):
        oracle.qgemm(huge, huge, [1.0], [1.0])


def test_int4_packing_order_round_trip_and_w4_equals_w8():
    assert oracle.pack4(np.array([-7, 3], np.int8)).tolist() == [0x39]
    assert oracle.unpack4(np.array([0x39, 0x8F], np.uint8)).tolist() == [-7, 3, -1, -8]
    pairs = np.array([(i, j) for i in range(-7, 8) for j in range(-7, 8)], np.int8)
    np.testing.assert_array_equal(oracle.unpack4(oracle.pack4(pairs)), pairs)
    r = rng(14)
    a = r.integers(-127, 128, (9, 26)).astype(np.int8)
    w = r.integers(-7, 8, (11, 26)).astype(np.int8)
    y8, acc8 = oracle.qgemm(a, w, [0.01], [0.3])
    y4, acc4 = oracle.qgemm(a, oracle.pack4(w), [0.01], [0.3], w_storage_bits=4)
    np.testing.assert_array_equal(acc4, acc8)
    np.testing.assert_array_equal(y4, y8)
    # fake_quant's packed output is the packing of its own codes
    x = r.standard_normal((6, 10)).astype(np.float32)
    m = oracle.absmax(x, PER_ROW)
    for b in (2, 3, 4):
        _, c, p = oracle.fake_quant(x, m, b, PER_ROW, want_packed4=True)
        np.testing.assert_array_equal(p, oracle.pack4(c))


def test_quantized_layer_tracks_the_float_layer():
    r = rng(15)
    x = r.standard_normal((48, 256)).astype(np.float32)
    w = (0.05 * r.standard_normal((32, 256))).astype(np.float32)
    mx, mw = oracle.absmax(x), oracle.absmax(w, PER_ROW)
    _, cx, _ = oracle.fake_quant(x, mx, 8)
    _, cw, _ = oracle.fake_quant(w, mw, 8, PER_ROW)
    y, _ = oracle.qgemm(cx, cw, oracle.scale_from_absmax(mx, 8), oracle.scale_from_absmax(mw, 8),
                        w_gran=PER_ROW)
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    rel = np.linalg.norm(y - ref) / np.linalg.norm(ref)
    # predicted from the two tensors' relative quantization errors (independent errors add)
    ex = math.sqrt(oracle.quant_error(x, mx, 8, 8)[0, 0]) / np.linalg.norm(x)
    ew = math.sqrt(oracle.quant_error(w, mw, 8, 8, PER_ROW).sum()) / np.linalg.norm(w)
    pred = math.hypot(ex, ew)
    assert 0.5 * pred < rel < 1.5 * pred


def test_sse_pair_against_numpy():
    r = rng(16)
    a = r.standard_normal(10_000).astype(np.float32)
    b = r.standard_normal(10_000).astype(np.float32)
    want = math.fsum(((a.astype(np.float64) - b.astype(np.float64)) ** 2).tolist())
    assert oracle.sse_pair(a, b) == pytest.approx(want, rel=1e-12)
    assert oracle.sse_pair(a, a) == 0.0


# ------------------------------------------------------------------------------- activations
def test_oracle_gelu_is_x_times_the_gaussian_distribution_function():
    """Pin of the oracle's activation against scipy's normal CDF (a different routine than erfc)."""
    from scipy.stats import norm
    x = np.linspace(-9, 9, 2001).astype(np.float32)
    want = (x.astype(np.float64) * norm.cdf(x.astype(np.float64))).astype(np.float32)
    np.testing.assert_array_equal(oracle.activation(x, oracle.ACT_GELU), want)
    np.testing.assert_array_equal(oracle.activation(x, oracle.ACT_RELU), np.maximum(x, 0))
    np.testing.assert_array_equal(oracle.activation(x, oracle.ACT_NONE), x)
