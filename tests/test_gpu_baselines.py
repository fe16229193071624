"""GPU parity: refined greedy approximation and the relative mean squared error (Sec. 2,
Tables 1-2) against the CPU oracle, through the C ABI."""
import numpy as np
import pytest

import oracle
from gpu_util import assert_coef_close, host, planes_host, to_dev, unpack_bits
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


def check_refined(W, k, planes_g, alpha_g):
    """Codes bit-exact; a differing entry is accepted only where the residual that decided it is a
    binary32 near-zero (within 1e-5 of the largest coefficient), and such rows are exempt from the
    coefficient comparison.  Returns the number of differing entries."""
    planes_r, alpha_r = oracle.refined_greedy_rows(W, k)
    rows, n = W.shape
    full = np.unpackbits(np.ascontiguousarray(planes_g).view(np.uint8).reshape(k, rows, -1), axis=2,
                         bitorder="little")
    assert not full[:, :, n:].any(), "pad bits must be zero"
    flips = 0
    clean = np.ones(rows, bool)
    if not np.array_equal(planes_g, planes_r):
        bg, br = unpack_bits(planes_g, n), unpack_bits(planes_r, n)
        for r in np.nonzero((bg != br).any(axis=(0, 2)))[0]:
            clean[r] = False
            j = int(np.nonzero((bg[:, r] != br[:, r]).any(axis=1))[0][0])   # first plane that differs
            B = br[:j, r].astype(np.float64).T * 2 - 1
            res = W[r].astype(np.float64)
            if j:
                res = res - B @ np.linalg.lstsq(B, res, rcond=None)[0]
            bad = np.nonzero(bg[j, r] != br[j, r])[0]
            assert np.abs(res[bad]).max() <= 1e-5 * np.abs(alpha_r[r]).max(), "row %d: not a near-tie" % r
            flips += len(bad)
    assert_coef_close(alpha_g[clean], alpha_r[clean], "alpha")
    return flips


@pytest.mark.parametrize("rows,n,k", [(5, 70, 1), (9, 300, 2), (33, 1024, 3), (3, 129, 4), (7, 4096, 2),
                                      (2, 5000, 3), (2, 16384, 4), (1200, 600, 2), (1500, 100, 3)])
def test_refined_greedy(amq, rows, n, k):
    g = np.random.default_rng(rows * 7 + n + k)
    W = (g.standard_normal((rows, n)) * 0.05).astype(np.float32)
    W[0, : min(n, 40)] = 0.0                     # a stretch of exact zeros (sign(0) = +1)
    say("refined greedy rows=%d n=%d k=%d" % (rows, n, k))
    pg, ag = amq.quantize_refined_greedy(to_dev(W), k)
    flips = check_refined(W, k, planes_host(pg), host(ag))
    say("  differing entries:", flips)


def test_refined_greedy_degenerate_rows(amq):
    W = np.zeros((4, 200), np.float32)
    W[1] = 0.75                                   # planes 1 and 2 coincide: singular Gram matrix
    W[2, ::2] = 1.0
    W[2, 1::2] = -1.0                             # exactly representable with one plane
    W[3] = np.linspace(-1, 1, 200, dtype=np.float32)
    pg, ag = amq.quantize_refined_greedy(to_dev(W), 3)
    assert check_refined(W, 3, planes_host(pg), host(ag)) == 0
    pr, ar = oracle.refined_greedy_rows(W, 3)
    assert np.array_equal(host(ag), ar)


def test_refined_greedy_strided_rows(amq):
    g = np.random.default_rng(77)
    big = (g.standard_normal((6, 700)) * 0.1).astype(np.float32)
    d = to_dev(big)[:, 100:400]                   # row stride 700, 300 columns
    pg, ag = amq.quantize_refined_greedy(d, 2)
    assert check_refined(np.ascontiguousarray(big[:, 100:400]), 2, planes_host(pg), host(ag)) == 0


@pytest.mark.parametrize("rows,n,k", [(7, 300, 2), (130, 1024, 3), (3, 129, 4), (1, 5000, 1), (1200, 600, 2)])
def test_relative_mse(amq, rows, n, k):
    g = np.random.default_rng(rows + n + k)
    W = (g.standard_normal((rows, n)) * 0.05).astype(np.float32)
    planes, alpha = oracle.quantize_rows(W, k, 2)
    say("relative mse rows=%d n=%d k=%d" % (rows, n, k))
    ratio, row_err, row_norm = oracle.relative_mse(W, planes, alpha)
    res, ge, gn = amq.relative_mse(to_dev(W), to_dev(planes), to_dev(alpha))
    res = host(res)
    assert np.allclose(host(ge), row_err, rtol=1e-10, atol=0)
    assert np.allclose(host(gn), row_norm, rtol=1e-10, atol=0)
    assert abs(res[2] - ratio) <= 1e-10 * ratio
    assert abs(res[0] - row_err.sum()) <= 1e-10 * row_err.sum()
    assert abs(res[1] - row_norm.sum()) <= 1e-10 * row_norm.sum()


def test_method_order_on_gpu_matches_the_tables(amq):
    """Greedy > Refined > Alternating in relative MSE for 2, 3, 4 bits (the order of Tables 1-2),
    computed entirely by the GPU path on LSTM-shaped Gaussian weights and on heavy-tailed weights,
    and each value equal to the oracle's."""
    g = np.random.default_rng(9)
    for W in ((g.standard_normal((1200, 600)) * 0.05).astype(np.float32), inputs.heavy_tailed(rows=256, cols=4096)):
        d = to_dev(W)
        for k in (2, 3, 4):
            vals = []
            for name, (pg, ag), (pr, ar) in (
                    ("greedy", amq.quantize_weights(d, k, 0), oracle.quantize_rows(W, k, 0)),
                    ("refined", amq.quantize_refined_greedy(d, k), oracle.refined_greedy_rows(W, k)),
                    ("alternating", amq.quantize_weights(d, k, 2), oracle.quantize_rows(W, k, 2))):
                got = float(host(amq.relative_mse(d, pg, ag)[0])[2])
                ref = oracle.relative_mse(W, pr, ar)[0]
                say("  %s k=%d: gpu %.6f oracle %.6f" % (name, k, got, ref))
                assert abs(got - ref) <= 1e-5 * ref
                vals.append(got)
            assert vals[0] > vals[1] > vals[2]
