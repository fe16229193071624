"""Pins of the oracle's ternary quantizer (the 2-bit case with alpha_1 = alpha_2, Sec. 2): library
least squares, brute-force nearest level, alternating-minimisation invariants, special cases that
reduce to 1-bit quantization, and the Gaussian fixed point in closed form.  CPU only."""
import math

import numpy as np
import pytest
from scipy.optimize import brentq
from scipy.stats import norm

import oracle


def tern(code):
    """t in {-1, 0, +1} from the two planes; also checks the plane convention of a zero."""
    b = code.astype(np.int64) * 2 - 1
    t = (b[0] + b[1]) // 2
    zero = t == 0
    assert np.array_equal(code[0][zero], np.ones(zero.sum(), np.uint8))     # 0 is stored as (+1, -1)
    assert np.array_equal(code[1][zero], np.zeros(zero.sum(), np.uint8))
    return t


def test_coefficients_are_equal_and_reconstruction_is_three_levels():
    g = np.random.default_rng(0)
    w = g.standard_normal(400).astype(np.float32)
    for T in range(4):
        code, alpha = oracle.ternary(w, T)
        assert alpha[0] == alpha[1] and alpha[0] > 0
        rec = oracle.dequantize(np.stack([np.packbits(np.pad(code[i], (0, 512 - 400)), bitorder="little")
                                          .view("<u4").astype(np.uint32)[None, :] for i in range(2)]),
                                alpha[None, :], 400)[0]
        a = np.float32(alpha[0] + alpha[1])
        assert np.array_equal(rec, a * tern(code).astype(np.float32))


def test_t0_is_the_threshold_rule_with_its_least_squares_coefficient():
    g = np.random.default_rng(1)
    for n in (7, 64, 301):
        w = g.standard_normal(n).astype(np.float32)
        code, alpha = oracle.ternary(w, 0)
        t = tern(code)
        w64 = w.astype(np.float64)
        thr = 0.7 * np.abs(w64).sum() / n
        safe = np.abs(np.abs(w64) - thr) > 1e-6
        assert np.array_equal(t[safe], (np.sign(w64) * (np.abs(w64) > thr))[safe].astype(np.int64))
        a = np.linalg.lstsq(t[:, None].astype(np.float64), w64, rcond=None)[0][0]    # library least squares
        assert abs(float(alpha[0]) + float(alpha[1]) - a) < 1e-6 * max(1.0, abs(a))


@pytest.mark.parametrize("T", [1, 2, 3, 5])
def test_codes_are_nearest_levels_and_coefficient_fits_the_previous_codes(T):
    """After T cycles: the codes are the nearest of {-a, 0, a} (brute force over the three levels),
    and a is the least-squares coefficient of the codes of cycle T - 1."""
    g = np.random.default_rng(10 + T)
    w = (g.standard_normal(257) * 1.7).astype(np.float32)
    code, alpha = oracle.ternary(w, T)
    prev_code, _ = oracle.ternary(w, T - 1)
    a = float(alpha[0]) + float(alpha[1])
    w64 = w.astype(np.float64)
    levels = np.array([-a, 0.0, a])
    nearest = np.abs(w64[:, None] - levels[None, :]).argmin(axis=1) - 1
    safe = np.abs(np.abs(w64) - a / 2) > 1e-6
    assert np.array_equal(tern(code)[safe], nearest[safe])
    tp = tern(prev_code).astype(np.float64)
    ls = np.linalg.lstsq(tp[:, None], w64, rcond=None)[0][0]
    assert abs(a - ls) < 1e-6 * max(1.0, abs(ls))


def test_error_never_increases_over_cycles():
    """Each half cycle minimises ||w - a t||^2 over its own variable, so the error of (a_T, codes_T) with
    a refit cannot exceed that of the cycle before."""
    g = np.random.default_rng(3)
    for trial in range(5):
        w = (g.standard_normal(500) * (1 + trial)).astype(np.float32).astype(np.float64)
        errs = []
        for T in range(5):
            code, _ = oracle.ternary(w.astype(np.float32), T)
            t = tern(code).astype(np.float64)
            a = (t @ w) / max(t @ t, 1.0)
            errs.append(((w - a * t) ** 2).sum())
        assert all(errs[i + 1] <= errs[i] * (1 + 1e-9) for i in range(4)), errs


def test_constant_magnitude_reduces_to_one_bit_quantization():
    """|w_l| = c for every l: nothing is zeroed, the result is Eq. 3 (sign, mean magnitude)."""
    g = np.random.default_rng(4)
    s = np.where(g.random(333) < 0.5, -1.0, 1.0)
    w = (0.375 * s).astype(np.float32)
    code1, alpha1 = oracle.greedy(w, 1)
    for T in (0, 1, 2):
        code, alpha = oracle.ternary(w, T)
        assert np.array_equal(code[0], code1[0]) and np.array_equal(code[1], code1[0])
        assert np.float32(alpha[0] + alpha[1]) == alpha1[0] == np.float32(0.375)


def test_three_level_input_is_reproduced_exactly():
    g = np.random.default_rng(5)
    t = g.integers(-1, 2, 1000)
    w = (0.8125 * t).astype(np.float32)
    for T in (0, 1, 2):
        code, alpha = oracle.ternary(w, T)
        assert np.array_equal(tern(code), t)
        assert np.float32(alpha[0] + alpha[1]) == np.float32(0.8125)


def test_all_zero_vector():
    code, alpha = oracle.ternary(np.zeros(130, np.float32), 2)
    assert alpha[0] == 0 and alpha[1] == 0
    assert np.array_equal(tern(code), np.zeros(130, np.int64))


def test_gaussian_fixed_point():
    """For w ~ N(0, 1) the alternating cycles converge to a = E[|w| : |w| > a / 2]
    = pdf(a/2) / (1 - cdf(a/2)); with n = 400000 entries the sample value is within 1 % of the root."""
    root = brentq(lambda a: a - norm.pdf(a / 2) / (1.0 - norm.cdf(a / 2)), 0.5, 3.0)
    w = np.random.default_rng(6).standard_normal(400000).astype(np.float32)
    _, alpha = oracle.ternary(w, 30)
    a = float(alpha[0]) + float(alpha[1])
    assert abs(a - root) < 0.01 * root, (a, root)
    # and one cycle from the threshold rule already moves towards it from the rule's own value
    a0 = float(sum(oracle.ternary(w, 0)[1]))
    thr = 0.7 * math.sqrt(2 / math.pi)
    assert abs(a0 - norm.pdf(thr) / (1.0 - norm.cdf(thr))) < 0.01 * a0


def test_rows_packing_matches_single_vectors():
    g = np.random.default_rng(7)
    W = g.standard_normal((9, 200)).astype(np.float32)
    planes, alpha = oracle.ternary_rows(W, 2)
    for r in range(9):
        code, al = oracle.ternary(W[r], 2)
        assert np.array_equal(alpha[r], al)
        for i in range(2):
            bits = np.unpackbits(planes[i, r].view(np.uint8), bitorder="little")
            assert np.array_equal(bits[:200], code[i]) and not bits[200:].any()
