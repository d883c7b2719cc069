"""Pins of the oracle's Hutchinson trace probe (Sec. 3.2.3) for a linear layer under a
mean-squared-error loss, and the GPU parity of mpq_rademacher / mpq_hutchinson_quad."""
import itertools
import os

import numpy as np
import pytest

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


# ------------------------------------------------------------------------------- oracle pins (CPU)
def test_hand_example_from_the_golden_file():
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "hutchinson_hand_example.txt")) if l[0] not in "#\n"]
    v = np.array([[float(a), float(b)] for a, b, _ in rows], np.float32)
    want = np.array([float(q) for _, _, q in rows])
    x = np.array([[1, 2], [3, 4]], np.float32)
    np.testing.assert_array_equal(oracle.hutchinson_quad(x, v), want)
    est, _ = oracle.hutchinson_trace(x, v)
    assert est == 30.0


@pytest.mark.parametrize("mk", [(5, 3), (17, 8), (3, 10)])
def test_mean_over_all_sign_vectors_is_the_frobenius_norm(mk):
    """E_v[v' A v] = Tr(A) holds exactly for the uniform distribution over all 2^K sign vectors:
    the enumeration turns the expectation into a finite mean.  A wrong index, a transposed operand
    or a missing square breaks it."""
    M, K = mk
    x = rng(1).standard_normal((M, K)).astype(np.float32)
    v = np.array(list(itertools.product([1.0, -1.0], repeat=K)), np.float32)
    q = oracle.hutchinson_quad(x, v)
    fro = float((x.astype(np.float64) ** 2).sum())
    assert q.mean() == pytest.approx(fro, rel=1e-12)
    est, _ = oracle.hutchinson_trace(x, v)
    assert est == pytest.approx(2.0 / M * fro, rel=1e-12)      # the exact trace of (2/(MN)) I (x) X'X


def test_special_probes():
    x = rng(2).standard_normal((40, 12)).astype(np.float32)
    xd = x.astype(np.float64)
    eye = np.eye(12, dtype=np.float32)
    np.testing.assert_allclose(oracle.hutchinson_quad(x, eye), (xd ** 2).sum(axis=0), rtol=1e-13)  # column norms
    ones = np.ones((1, 12), np.float32)
    assert oracle.hutchinson_quad(x, ones)[0] == pytest.approx((xd.sum(axis=1) ** 2).sum(), rel=1e-13)
    # an orthonormal X (first K columns of the identity): every sign vector has ||X v||^2 = K
    q = oracle.hutchinson_quad(np.eye(16, 12, dtype=np.float32), oracle.rademacher(3, 0, 9, 12))
    np.testing.assert_array_equal(q, np.full(9, 12.0))
    # scaling a probe by c scales its quadratic form by c^2; a non-square, asymmetric case catches a transposed v
    v = rng(4).standard_normal((3, 12)).astype(np.float32)
    np.testing.assert_allclose(oracle.hutchinson_quad(x, 2 * v), 4 * oracle.hutchinson_quad(x, v), rtol=1e-13)
    np.testing.assert_allclose(oracle.hutchinson_quad(x, v), ((xd @ v.astype(np.float64).T) ** 2).sum(axis=0), rtol=1e-12)


def test_rademacher_bits_come_from_the_philox_words_as_documented():
    """The generator itself is pinned by the published known-answer vectors; this pins the layout:
    element e -> block e / 128, word (e % 128) / 32, bit e % 32, set bit = -1, key word 1 tagged."""
    seed, sid = 0x0123456789ABCDEF, 0xFEDCBA9876543210
    rows, cols = 7, 100                      # 700 elements: 5.47 blocks, rows that straddle blocks
    v = oracle.rademacher(seed, sid, rows, cols).ravel()
    assert set(np.unique(v)) == {-1.0, 1.0}
    key = (seed & 0xFFFFFFFF, (seed >> 32) ^ 0x5241444D)
    for e in (0, 1, 31, 32, 127, 128, 129, 255, 256, 511, 640, 699):
        g = e >> 7
        w = oracle.philox4x32_10((g & 0xFFFFFFFF, g >> 32, sid & 0xFFFFFFFF, sid >> 32), key)
        bit = (int(w[(e & 127) >> 5]) >> (e & 31)) & 1
        assert v[e] == (-1.0 if bit else 1.0), e
    # the element index is r * cols + c: a different shape with the same count gives the same stream
    np.testing.assert_array_equal(oracle.rademacher(seed, sid, 100, 7).ravel(), v)
    # other stream, other seed: different draws
    assert (oracle.rademacher(seed, sid + 1, rows, cols).ravel() != v).mean() > 0.4
    assert (oracle.rademacher(seed + 1, sid, rows, cols).ravel() != v).mean() > 0.4


def test_rademacher_statistics_and_the_estimator_moments():
    """Signs are balanced and uncorrelated, so the estimator is unbiased and has the variance of
    independent random signs, Var(v' A v) = 2 (||A||_F^2 - sum_i A_ii^2) with A = X'X."""
    P, K, M = 4096, 24, 50
    v = oracle.rademacher(11, 5, P, K)
    assert abs(v.mean()) < 4 / np.sqrt(P * K)
    corr = (v.astype(np.float64).T @ v.astype(np.float64)) / P          # K x K, identity in expectation
    assert np.abs(corr - np.eye(K)).max() < 5 / np.sqrt(P)
    x = rng(6).standard_normal((M, K)).astype(np.float32)
    q = oracle.hutchinson_quad(x, v)
    a = x.astype(np.float64).T @ x.astype(np.float64)
    tr = np.trace(a)
    var = 2.0 * ((a ** 2).sum() - (np.diag(a) ** 2).sum())
    assert abs(q.mean() - tr) < 4 * np.sqrt(var / P)
    assert q.var(ddof=1) == pytest.approx(var, rel=0.15)
    est, err = oracle.hutchinson_trace(x, v)
    assert abs(est - 2.0 / M * tr) < 4 * err
    assert err == pytest.approx(2.0 / M * np.sqrt(var / P), rel=0.1)


# ---------------------------------------------------------------------------------- GPU parity
def _torch():
    import torch
    return torch


def dev(a):
    return _torch().from_numpy(np.ascontiguousarray(a)).cuda()


def dev_misaligned(a):
    """The same values at an address that is 4-byte but not 16-byte aligned."""
    t = _torch()
    a = np.ascontiguousarray(a)
    buf = t.empty(a.size + 1, dtype=t.from_numpy(a).dtype, device="cuda")
    view = buf[1:].view(a.shape)
    view.copy_(t.from_numpy(a))
    return view


@pytest.mark.gpu
@pytest.mark.parametrize("shape", [(1, 1), (1, 31), (7, 100), (32, 1024), (33, 1000), (128, 4096), (3, 129)])
def test_gpu_rademacher_bit_exact(shape):
    from paper_2302_01382_amd import mpq
    t = _torch()
    seed, sid = 0x9E3779B97F4A7C15, 3
    want = oracle.rademacher(seed, sid, *shape)
    got = mpq.rademacher(seed, sid, *shape)
    np.testing.assert_array_equal(got.cpu().numpy(), want)
    buf = t.zeros(shape[0] * shape[1] + 2, dtype=t.float32, device="cuda")
    mpq.rademacher(seed, sid, *shape, out=buf[1:-1])
    host = buf.cpu().numpy()
    np.testing.assert_array_equal(host[1:-1], want.ravel())
    assert host[0] == 0 and host[-1] == 0          # nothing written outside the tensor


@pytest.mark.gpu
@pytest.mark.parametrize("mkp", [(64, 256, 32), (33, 31, 5), (1, 4, 1), (1000, 100, 40), (300, 70, 130), (4100, 1024, 64),
                                 (2085, 2048, 96), (515, 36, 257), (40000, 64, 32), (100, 96, 70), (37, 16, 3), (200, 1008, 33), (100, 48, 5), (64, 40, 8)])
def test_gpu_hutchinson_quad_matches_the_oracle(mkp):
    from paper_2302_01382_amd import mpq
    M, K, P = mkp
    x = rng(20).standard_normal((M, K)).astype(np.float32)
    v = oracle.rademacher(21, 0, P, K)
    want = oracle.hutchinson_quad(x, v)
    for mk in (dev, dev_misaligned):
        got = mpq.hutchinson_quad(mk(x), mk(v)).cpu().numpy()
        np.testing.assert_allclose(got, want, rtol=1e-4, atol=0)
    # arbitrary real probes go through the same contraction
    g = rng(22).standard_normal((P, K)).astype(np.float32)
    np.testing.assert_allclose(mpq.hutchinson_quad(dev(x), dev(g)).cpu().numpy(), oracle.hutchinson_quad(x, g), rtol=1e-4)
    # the sign probes drawn inside the kernel: the same bits as the stored matrix (k is summed in
    # another order, so the fp32 sums agree to rounding, not bit for bit)
    if K % 16 == 0:
        a = mpq.hutchinson_quad_signs(dev(x), 21, 0, P).cpu().numpy()
        np.testing.assert_allclose(a, want, rtol=1e-4, atol=0)
        np.testing.assert_allclose(a, mpq.hutchinson_quad(dev(x), mpq.rademacher(21, 0, P, K)).cpu().numpy(), rtol=2e-5)
        np.testing.assert_array_equal(a, mpq.hutchinson_quad_signs(dev(x), 21, 0, P).cpu().numpy())
    else:
        with pytest.raises(mpq.MpqError):
            mpq.hutchinson_quad_signs(dev(x), 21, 0, P)
    # reproducible bit for bit, and zero for a zero tensor
    a = mpq.hutchinson_quad(dev(x), dev(v)).cpu().numpy()
    np.testing.assert_array_equal(a, mpq.hutchinson_quad(dev(x), dev(v)).cpu().numpy())
    assert not mpq.hutchinson_quad(dev(np.zeros_like(x)), dev(v)).cpu().numpy().any()


@pytest.mark.gpu
def test_gpu_trace_estimate_full_size_against_oracle_and_closed_form():
    """Configuration 5's activation tensor (16384 x 1024) with 32 probes: the same probes on both
    sides (bit-exact signs), the estimate within 1e-4 of the oracle's and within four standard
    errors of the exact trace (2 / M) ||X||_F^2."""
    from paper_2302_01382_amd import hessian, mpq, workloads
    x, _, _ = workloads.cfg5_tensors()
    M, K = x.shape
    est, err = hessian.trace_linear_mse(dev(x), probes=32, seed=5, stream_id=9)
    v = oracle.rademacher(5, 9, 32, K)
    est_o, err_o = oracle.hutchinson_trace(x, v)
    assert est == pytest.approx(est_o, rel=1e-4)
    assert err == pytest.approx(err_o, rel=1e-3)
    exact = 2.0 / M * float((x.astype(np.float64) ** 2).sum())
    assert abs(est - exact) < 4 * err
    # ordering a few tensors of different energy: the order follows the exact traces
    ts = [dev((s * x[:4096]).astype(np.float32)) for s in (1.0, 0.25, 2.0)]
    order, traces = hessian.order_by_trace(ts, probes=32, seed=1)
    assert order == [1, 0, 2]
