"""GPU parity: ternary quantization as the 2-bit case with equal coefficients (Sec. 2) against the
CPU oracle, through the C ABI; and the result consumed by the 2-bit product path."""
import numpy as np
import pytest

import oracle
from gpu_util import assert_coef_close, assert_vec_close, host, planes_host, to_dev, unpack_bits
from paper_1802_00150_amd import inputs

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


@pytest.fixture(scope="module")
def amq():
    import paper_1802_00150_amd as m
    m.binding.lib()
    return m


@pytest.fixture(autouse=True)
def threads():
    oracle.set_threads(oracle.host_threads())
    yield
    oracle.set_threads(1)


def check_ternary(W, T, planes_g, alpha_g):
    """Codes bit-exact; a differing entry is accepted only where |w| is a binary32 near-tie at the
    threshold that decided it (half the oracle's coefficient sum for T > 0, the 0.7 mean for T = 0),
    and such rows are exempt from the coefficient comparison.  Returns the number of differing entries."""
    planes_r, alpha_r = oracle.ternary_rows(W, T)
    rows, n = W.shape
    full = np.unpackbits(np.ascontiguousarray(planes_g).view(np.uint8).reshape(2, rows, -1), axis=2,
                         bitorder="little")
    assert not full[:, :, n:].any(), "pad bits must be zero"
    assert np.array_equal(alpha_g[:, 0], alpha_g[:, 1])
    flips = 0
    clean = np.ones(rows, bool)
    if not np.array_equal(planes_g, planes_r):
        bg, br = unpack_bits(planes_g, n), unpack_bits(planes_r, n)
        for r in np.nonzero((bg != br).any(axis=(0, 2)))[0]:
            clean[r] = False
            w = np.abs(W[r].astype(np.float64))
            thr = 0.7 * w.sum() / n if T == 0 else float(alpha_r[r, 0]) + 0.0   # a / 2 = alpha_1
            bad = np.nonzero((bg[:, r] != br[:, r]).any(axis=0))[0]
            assert np.abs(w[bad] - thr).max() <= 1e-5 * max(thr, 1e-30), "row %d: not a near-tie" % r
            flips += len(bad)
    assert_coef_close(alpha_g[clean], alpha_r[clean], "alpha")
    return flips


@pytest.mark.parametrize("rows,n", [(5, 70), (9, 300), (33, 1024), (3, 129), (7, 4096), (2, 16384), (1500, 640),
                                    (1100, 4096)])
@pytest.mark.parametrize("T", [0, 1, 2, 4])
def test_ternary(amq, rows, n, T):
    g = np.random.default_rng(rows * 11 + n + T)
    W = (g.standard_normal((rows, n)) * 0.05).astype(np.float32)
    W[0, : min(n, 40)] = 0.0                      # a stretch of exact zeros
    say("ternary rows=%d n=%d T=%d" % (rows, n, T))
    pg, ag = amq.quantize_ternary(to_dev(W), T)
    flips = check_ternary(W, T, planes_host(pg), host(ag))
    say("  differing entries:", flips)
    assert flips <= max(2, rows * n // 100000)


def test_ternary_degenerate_and_strided_rows(amq):
    W = np.zeros((5, 200), np.float32)
    W[1] = 0.75                                   # constant magnitude: nothing is zeroed
    W[2, ::2] = 1.0
    W[2, 1::2] = -1.0
    W[3] = np.linspace(-1, 1, 200, dtype=np.float32)
    W[4, 17] = -3.0                               # a single non-zero entry
    for T in (0, 2):
        pg, ag = amq.quantize_ternary(to_dev(W), T)
        assert check_ternary(W, T, planes_host(pg), host(ag)) == 0
        assert np.array_equal(host(ag), oracle.ternary_rows(W, T)[1])
    g = np.random.default_rng(78)
    big = (g.standard_normal((6, 700)) * 0.1).astype(np.float32)
    d = to_dev(big)[:, 100:400]                   # row stride 700, 300 columns
    pg, ag = amq.quantize_ternary(d, 2)
    assert check_ternary(np.ascontiguousarray(big[:, 100:400]), 2, planes_host(pg), host(ag)) == 0


def test_ternary_weights_in_the_two_bit_product(amq):
    """The two planes and equal coefficients go through the product path unchanged: the GPU product on
    GPU-quantized ternary weights equals the oracle's product on oracle-quantized ones."""
    g = np.random.default_rng(5)
    m, n, batch = 700, 1024, 24
    W = (g.standard_normal((m, n)) * 0.02).astype(np.float32)
    X = g.standard_normal((batch, n)).astype(np.float32)
    pg, ag = amq.quantize_ternary(to_dev(W), 2)
    Wp, alpha = oracle.ternary_rows(W, 2)
    assert np.array_equal(planes_host(pg), Wp)
    Xp, beta = oracle.quantize_rows(X, 2, 2)
    Y = amq.binary_gemm(pg, ag, n, to_dev(Xp), to_dev(beta))
    assert_vec_close(host(Y), oracle.binary_gemm(Wp, alpha, n, Xp, beta))
    # and its error sits between 1-bit and unconstrained 2-bit alternating quantization
    e1 = oracle.relative_mse(W, *oracle.quantize_rows(W, 1, 2))[0]
    e2 = oracle.relative_mse(W, *oracle.quantize_rows(W, 2, 2))[0]
    et = float(host(amq.relative_mse(to_dev(W), pg, ag)[0])[2])
    say("  relative mse: 1-bit %.4f ternary %.4f 2-bit %.4f" % (e1, et, e2))
    assert e2 < et < e1
