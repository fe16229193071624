"""Pins for the oracle's quantizer (greedy, least squares, code table, BST, Alg. 2).

Each test checks the oracle against something other than itself: a closed form,
a textbook/library routine, brute force on tiny inputs, a value the paper
prints, or an invariant that the mathematics fixes.
"""
import itertools
import math

import numpy as np
import pytest
from scipy import integrate, stats

import oracle
from conftest import read_golden


def signs(code):
    return code.astype(np.float64) * 2.0 - 1.0


def recon(code, alpha):
    return (signs(code) * np.asarray(alpha, np.float64)[:, None]).sum(0)


def patterns(k):
    """All 2^k sign vectors, row p has s_i = +1 iff bit (k-i) of p is set."""
    return np.array([[1.0 if (p >> (k - i)) & 1 else -1.0 for i in range(1, k + 1)] for p in range(1 << k)])


# ---------------------------------------------------------------- greedy (Eq. 3-4)

def test_greedy_gaussian_closed_forms():
    # For w ~ N(0, s^2): alpha_1 = E|w| = s*sqrt(2/pi); relative error 1 - 2/pi.
    # Second stage: alpha_2 = E| |w| - alpha_1 |, error E(| |w|-a1 | - a2)^2; by quadrature.
    s = 0.02
    n = 1 << 20
    w = (np.random.default_rng(1).standard_normal(n) * s).astype(np.float32)
    code, alpha = oracle.greedy(w, 3)
    a1 = math.sqrt(2 / math.pi)
    pdf = stats.norm.pdf
    a2 = 2 * integrate.quad(lambda z: abs(z - a1) * pdf(z), 0, 12, points=[a1])[0]
    a3 = 2 * integrate.quad(lambda z: abs(abs(z - a1) - a2) * pdf(z), 0, 12, points=[a1 - a2, a1, a1 + a2])[0]
    e2 = 2 * integrate.quad(lambda z: (abs(z - a1) - a2) ** 2 * pdf(z), 0, 12, points=[a1])[0]
    assert abs(alpha[0] / s - a1) < 3e-3
    assert abs(alpha[1] / s - a2) < 3e-3
    assert abs(alpha[2] / s - a3) < 3e-3
    ww = w.astype(np.float64)
    rel1 = ((ww - recon(code[:1], alpha[:1])) ** 2).sum() / (ww ** 2).sum()
    rel2 = ((ww - recon(code[:2], alpha[:2])) ** 2).sum() / (ww ** 2).sum()
    assert abs(rel1 - (1 - 2 / math.pi)) < 3e-3
    assert abs(rel2 - e2) < 3e-3
    # first plane is sign(w)
    assert np.array_equal(code[0], (w >= 0).astype(np.uint8))


def test_greedy_residual_signs_tiny_by_hand():
    # w = [3, -1, 1, -3]: alpha_1 = 2, b_1 = + - + -, r = [1, 1, -1, -1], alpha_2 = 1, b_2 = + + - -, r = 0.
    w = np.array([3, -1, 1, -3], np.float32)
    code, alpha = oracle.greedy(w, 2)
    assert alpha.tolist() == [2.0, 1.0]
    assert code.tolist() == [[1, 0, 1, 0], [1, 1, 0, 0]]
    assert oracle.error(w, code, alpha) == 0.0


def test_sign_of_zero_is_plus():
    w = np.array([0.0, -0.0, 1.0, -1.0], np.float32)
    code, alpha = oracle.greedy(w, 1)
    assert code[0].tolist() == [1, 1, 1, 0]
    assert alpha[0] == np.float32(0.5)


# ---------------------------------------------------------------- k = 1 closed form

@pytest.mark.parametrize("T", [0, 1, 2, 5])
def test_one_bit_closed_form_any_T(T):
    w = np.random.default_rng(T).standard_normal(777).astype(np.float32)
    code, alpha = oracle.quantize(w, 1, T)
    assert np.array_equal(code[0], (w >= 0).astype(np.uint8))
    assert abs(float(alpha[0]) - np.abs(w.astype(np.float64)).mean()) <= 1e-7 * float(alpha[0])


# ---------------------------------------------------------------- least squares (Eq. 5)

@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_ls_matches_library_lstsq(k):
    g = np.random.default_rng(10 + k)
    for n in (5, 33, 300, 1024):
        w = g.standard_normal(n).astype(np.float32)
        code = (g.random((k, n)) < 0.5).astype(np.uint8)
        Bm = signs(code).T
        if np.linalg.matrix_rank(Bm) < k:
            continue
        ref = np.linalg.lstsq(Bm, w.astype(np.float64), rcond=None)[0]
        a, ok = oracle.ls(w, code, np.zeros(k, np.float32))
        assert ok
        assert np.allclose(a, ref, rtol=2e-6, atol=1e-7)
        # normal equations: residual orthogonal to every plane
        res = w.astype(np.float64) - Bm @ a.astype(np.float64)
        assert np.all(np.abs(Bm.T @ res) <= 1e-5 * n * np.abs(w).max())


def test_ls_singular_keeps_coefficients():
    g = np.random.default_rng(3)
    w = g.standard_normal(40).astype(np.float32)
    b = (g.random(40) < 0.5).astype(np.uint8)
    keep = np.array([0.3, 0.1], np.float32)
    for code in (np.stack([b, b]), np.stack([b, 1 - b])):
        a, ok = oracle.ls(w, code, keep)
        assert not ok and np.array_equal(a, keep)
    # three planes with b3 = product of an exact dependency: b1, b2, b1 (dependent)
    c = (g.random(40) < 0.5).astype(np.uint8)
    a, ok = oracle.ls(w, np.stack([b, c, b]), np.array([1, 2, 3], np.float32))
    assert not ok and a.tolist() == [1, 2, 3]


def test_ls_nearly_singular_still_solved():
    # two planes that differ in one entry: Gram matrix has determinant 4(n-1) != 0
    n = 64
    g = np.random.default_rng(4)
    w = g.standard_normal(n).astype(np.float32)
    b = (g.random(n) < 0.5).astype(np.uint8)
    c = b.copy()
    c[7] ^= 1
    a, ok = oracle.ls(w, np.stack([b, c]), np.zeros(2, np.float32))
    ref = np.linalg.lstsq(signs(np.stack([b, c])).T, w.astype(np.float64), rcond=None)[0]
    assert ok and np.allclose(a, ref, rtol=1e-5)


# ---------------------------------------------------------------- code table and BST (Alg. 1)

def test_fig1_boundaries_golden():
    for a1, a2, *rest in read_golden("fig1_two_bit.txt"):
        v, pat, mid = oracle.code_table(np.array([a1, a2], np.float32))
        assert v.tolist() == rest[:4]
        assert mid.tolist() == rest[4:]


def test_code_table_is_sorted_with_fixed_tie_break():
    g = np.random.default_rng(5)
    for k in (1, 2, 3, 4):
        P = patterns(k)
        for trial in range(200):
            alpha = g.standard_normal(k).astype(np.float32)
            if trial % 5 == 0:
                alpha[g.integers(k)] = 0.0           # duplicate code values
            if trial % 7 == 0 and k > 1:
                alpha[0] = alpha[1]
            v, pat, mid = oracle.code_table(alpha)
            assert np.all(np.diff(v) >= 0)
            assert sorted(pat.tolist()) == list(range(1 << k))
            exact = P @ alpha.astype(np.float64)
            assert np.allclose(v, exact[pat], rtol=0, atol=4e-7 * np.abs(alpha).sum() + 1e-30)
            ties = np.diff(v) == 0
            assert np.all(np.diff(pat)[ties] > 0)
            assert np.all(np.diff(mid) >= 0)


@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_bst_equals_brute_force_nearest_code(k):
    # Sec. 3: the code of an entry is the one at least distance among all 2^k codes.
    g = np.random.default_rng(20 + k)
    P = patterns(k)
    for trial in range(300):
        n = int(g.integers(1, 65))
        alpha = g.standard_normal(k).astype(np.float32)
        mode = trial % 4
        if mode == 1:
            alpha = np.abs(alpha)                      # non-negative, unordered
        elif mode == 2:
            alpha = -np.sort(-np.abs(alpha))           # the paper's ordering assumption
        elif mode == 3 and k > 1:
            alpha[-1] = alpha[0]                       # equal coefficients
        w = (g.standard_normal(n) * 1.5 * np.abs(alpha).sum()).astype(np.float32)
        code = oracle.bst(w, alpha)
        values = P @ alpha.astype(np.float64)           # exact code values
        dist = np.abs(w.astype(np.float64)[:, None] - values[None, :])
        best = dist.min(1)
        got = np.abs(w.astype(np.float64) - recon(code, alpha))
        scale = np.abs(alpha).sum() + 1e-30
        assert np.all(got <= best + 1e-6 * scale)
        # where the nearest code is unique by a margin, the pattern itself must match
        order = np.sort(dist, 1)
        unique = (order[:, 1] - order[:, 0]) > 1e-5 * scale if k > 0 and (1 << k) > 1 else np.ones(n, bool)
        p_best = dist.argmin(1)
        p_got = np.zeros(n, int)
        for i in range(k):
            p_got |= code[i].astype(int) << (k - 1 - i)
        assert np.array_equal(p_got[unique], p_best[unique])


def test_bst_tie_goes_up():
    # Alg. 1 compares with ">=": an entry exactly on a boundary takes the upper code.
    alpha = np.array([0.75, 0.25], np.float32)      # boundaries -0.75, 0, 0.75
    w = np.array([-0.75, 0.0, 0.75, -0.7500001, 0.7499999], np.float32)
    code = oracle.bst(w, alpha)
    assert recon(code, alpha).tolist() == [-0.5, 0.5, 1.0, -1.0, 0.5]


def test_two_bit_closed_form():
    # Sec. 3 (end of the BST paragraph): for alpha_1 >= alpha_2 >= 0,
    # b_1 = sign(w), b_2 = sign(w - alpha_1 b_1).
    g = np.random.default_rng(6)
    for _ in range(200):
        a = np.sort(np.abs(g.standard_normal(2)))[::-1].astype(np.float32)
        w = (g.standard_normal(500) * 2).astype(np.float32)
        code = oracle.bst(w, a)
        b1 = w >= 0
        b2 = (w - a[0] * np.where(b1, np.float32(1), np.float32(-1))) >= 0
        assert np.array_equal(code[0], b1.astype(np.uint8))
        assert np.array_equal(code[1], b2.astype(np.uint8))


# ---------------------------------------------------------------- Alg. 2 as a whole

@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_error_never_increases(k):
    # Each half-step minimises Eq. 2 exactly over its own block of unknowns.
    g = np.random.default_rng(30 + k)
    for n in (1, 2, 7, 64, 300, 1024, 4096):
        for dist in range(3):
            w = g.standard_normal(n)
            if dist == 1:
                w = w ** 3
            if dist == 2:
                w = np.abs(w)                      # one-sided data: coefficients can go unordered
            w = w.astype(np.float32)
            T = 4
            code, alpha, tr = oracle.quantize(w, k, T, trace=True)
            tol = 1e-6 * float((w.astype(np.float64) ** 2).sum()) + 1e-30
            assert np.all(np.diff(tr) <= tol), (n, dist, tr)
            assert tr[-1] <= tr[0] + tol          # alternating <= greedy
            # the trace is the objective of the state the oracle reports at that point
            c0, a0 = oracle.greedy(w, k)
            assert tr[0] == oracle.error(w, c0, a0)
            a1, _ = oracle.ls(w, c0, a0)
            assert tr[1] == oracle.error(w, c0, a1)
            assert tr[-1] == oracle.error(w, code, alpha)


def test_alternating_composition_of_the_pinned_steps():
    # Alg. 2 is greedy, then T x (LS; BST), no trailing LS: rebuild from the pinned pieces.
    g = np.random.default_rng(8)
    for k in (2, 3, 4):
        w = g.standard_normal(515).astype(np.float32)
        c, a = oracle.greedy(w, k)
        for _ in range(2):
            a, _ = oracle.ls(w, c, a)
            c = oracle.bst(w, a)
        c2, a2 = oracle.quantize(w, k, 2)
        assert np.array_equal(c, c2) and np.array_equal(a, a2)


def lloyd_max_rel_mse(levels):
    """Lloyd-Max quantizer of N(0,1) with the given number of levels (textbook iteration)."""
    q = np.linspace(-1.5, 1.5, levels)
    for _ in range(2000):
        t = np.concatenate([[-np.inf], 0.5 * (q[1:] + q[:-1]), [np.inf]])
        mass = stats.norm.cdf(t[1:]) - stats.norm.cdf(t[:-1])
        q = (stats.norm.pdf(t[:-1]) - stats.norm.pdf(t[1:])) / mass
    return 1.0 - float((mass * q * q).sum())


def test_gaussian_two_bit_lands_between_lloyd_max_and_greedy():
    # Every symmetric 4-level set is +-a1 +-a2, so the 4-level Lloyd-Max error is a lower
    # bound for k = 2 and greedy is an upper bound; two cycles land in between.
    n = 1 << 18
    w = np.random.default_rng(9).standard_normal(n).astype(np.float32)
    ww = (w.astype(np.float64) ** 2).sum()
    lm4 = lloyd_max_rel_mse(4)
    assert abs(lm4 - 0.1175) < 5e-4
    _, _, tr = oracle.quantize(w, 2, 2, trace=True)
    assert lm4 - 2e-3 <= tr[-1] / ww < tr[0] / ww
    assert tr[-1] / ww < 0.1225
    _, _, tr = oracle.quantize(w, 2, 30, trace=True)
    assert abs(tr[-1] / ww - lm4) < 2e-3          # the iteration is Lloyd's algorithm here
    _, _, tr3 = oracle.quantize(w, 3, 2, trace=True)
    assert lloyd_max_rel_mse(8) - 2e-3 <= tr3[-1] / ww < tr3[0] / ww


def test_global_optimum_by_exhaustion_tiny():
    # n = 6, k = 2: enumerate all code matrices, solve LS for each; Alg. 2's result can
    # not beat the global optimum of Eq. 2 and must not be worse than greedy.
    g = np.random.default_rng(11)
    n, k = 6, 2
    for _ in range(5):
        w = g.standard_normal(n).astype(np.float32)
        best = np.inf
        for bits in itertools.product([0, 1], repeat=n * k):
            Bm = (np.array(bits, np.float64).reshape(k, n) * 2 - 1).T
            a, res, rank, _ = np.linalg.lstsq(Bm, w.astype(np.float64), rcond=None)
            e = float(((w - Bm @ a) ** 2).sum())
            best = min(best, e)
        code, alpha, tr = oracle.quantize(w, k, 3, trace=True)
        assert best - 1e-9 <= tr[-1] <= tr[0] + 1e-9


def test_zero_vector_and_constant_magnitude():
    # h_0 = 0 at the first time step: coefficients 0, all codes +1, Gram matrix singular.
    for k in (1, 2, 3):
        code, alpha = oracle.quantize(np.zeros(300, np.float32), k, 2)
        assert np.all(alpha == 0) and np.all(code == 1)
    w = np.array([0.5, -0.5, 0.5, 0.5, -0.5], np.float32)
    code, alpha, tr = oracle.quantize(w, 2, 2, trace=True)
    assert tr[-1] == 0.0 and np.all(np.diff(tr) <= 0)


def test_fixed_point_is_idempotent():
    w = np.random.default_rng(12).standard_normal(2048).astype(np.float32)
    c, a = oracle.quantize(w, 2, 60)
    a2, _ = oracle.ls(w, c, a)
    c2 = oracle.bst(w, a2)
    a3, _ = oracle.ls(w, c2, a2)
    assert np.array_equal(c2, oracle.bst(w, a3))


# ---------------------------------------------------------------- packing

def test_pack_matches_numpy_packbits():
    g = np.random.default_rng(13)
    for n in list(range(1, 131)) + [300, 1024, 4096]:
        bits = (g.random(n) < 0.5).astype(np.uint8)
        words = oracle.pack(bits)
        assert words.shape[0] == 4 * ((n + 127) // 128)
        ref = np.zeros(words.shape[0] * 32, np.uint8)
        ref[:n] = bits
        ref = np.packbits(ref, bitorder="little").view("<u4")
        assert np.array_equal(words, ref)


def test_quantize_rows_is_per_row_quantize_plus_pack():
    g = np.random.default_rng(14)
    W = g.standard_normal((9, 77)).astype(np.float32)
    planes, alpha = oracle.quantize_rows(W, 3, 2)
    for r in range(9):
        c, a = oracle.quantize(W[r], 3, 2)
        assert np.array_equal(alpha[r], a)
        for i in range(3):
            assert np.array_equal(planes[i, r], oracle.pack(c[i]))


# ---------------------------------------------------------------- cost model (Sec. 4)

def test_gamma_matches_printed_speedups():
    for m, n, kw, kh, printed in read_golden("gamma_sec4.txt"):
        assert abs(oracle.gamma(m, n, kw, kh) - printed) < 0.25
    # closed form retyped once, at a different shape, to catch a transposed m / n
    m, n, kw, kh = 42000.0, 1024.0, 2.0, 3.0
    ref = 2 * m * n / ((2 * kw * kh * m * n + 4 * kh * kh * n) / 32 + 6 * kh * n + 2 * kw * kh * m)
    assert abs(oracle.gamma(m, n, kw, kh) - ref) < 1e-12


def test_table6_ratios_are_self_consistent():
    rows = read_golden("table6_cpu_timing.txt")
    fp = {int(r[0]): r[3] for r in rows if r[2] == 0}
    for r in rows:
        if r[2] == 0:
            continue
        assert abs(fp[int(r[0])] / r[3] - r[6]) < 0.06
        assert abs(r[4] / r[3] - r[5]) < 0.006
