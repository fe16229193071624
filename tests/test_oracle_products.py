"""Pins for the oracle's binary products, quantized GEMM and the LSTM / GRU steps.

The references here are textbook dense products in binary64 on the de-quantized
operands (numpy matmul), written independently of the oracle's packed-code path.
"""
import numpy as np
import pytest

import oracle


def unpack(planes, n):
    """[k, rows, wpr] uint32 -> [k, rows, n] of +-1 (independent of the oracle: numpy unpackbits)."""
    k, rows, wpr = planes.shape
    bits = np.unpackbits(np.ascontiguousarray(planes).view(np.uint8).reshape(k, rows, wpr * 4), axis=2,
                         bitorder="little")
    assert np.all(bits[:, :, n:] == 0), "pad bits must be zero"
    return bits[:, :, :n].astype(np.int64) * 2 - 1


def dequant(planes, coef, n):
    """sum_i coef[:, i] * plane_i  -> [rows, n] float64."""
    s = unpack(planes, n).astype(np.float64)
    return np.einsum("irn,ri->rn", s, coef.astype(np.float64))


def rand_planes(g, k, rows, n):
    bits = (g.random((k, rows, n)) < 0.5).astype(np.uint8)
    return np.stack([np.stack([oracle.pack(bits[i, r]) for r in range(rows)]) for i in range(k)]), bits


def test_binary_dots_all_lengths_against_integer_matmul():
    g = np.random.default_rng(1)
    for n in list(range(1, 131)) + [300, 1024]:
        k_w, k_a, m, B = 2, 3, 5, 3
        Wp, wb = rand_planes(g, k_w, m, n)
        Xp, xb = rand_planes(g, k_a, B, n)
        D = oracle.binary_dots(Wp, n, Xp)
        ws = wb.astype(np.int64) * 2 - 1
        xs = xb.astype(np.int64) * 2 - 1
        ref = np.einsum("irn,jbn->brij", ws, xs)
        assert D.shape == (B, m, k_w, k_a)
        assert np.array_equal(D, ref)
        # App. A: product = XNOR then bit count, i.e. n - 2 * popcount(xor) on the packed words
        xor = Wp[:, None, :, None, :] ^ Xp[None, :, None, :, :]            # [k_w, k_a, m, B, wpr]
        pop = np.unpackbits(xor.view(np.uint8), axis=-1).sum(-1).astype(np.int64)
        assert np.array_equal(D, (n - 2 * pop).transpose(3, 2, 0, 1))


@pytest.mark.parametrize("k_w,k_a", [(1, 1), (2, 2), (2, 3), (3, 3), (4, 4)])
def test_gemm_equals_dense_product_of_dequantized(k_w, k_a):
    g = np.random.default_rng(2)
    m, n, B = 37, 300, 5
    W = (g.standard_normal((m, n)) * 0.05).astype(np.float32)
    X = g.standard_normal((B, n)).astype(np.float32)
    bias = (g.standard_normal(m) * 0.1).astype(np.float32)
    Wp, alpha = oracle.quantize_rows(W, k_w, 2)
    Xp, beta = oracle.quantize_rows(X, k_a, 2)
    ref = dequant(Xp, beta, n) @ dequant(Wp, alpha, n).T
    Y = oracle.binary_gemm(Wp, alpha, n, Xp, beta)
    assert np.allclose(Y, ref, rtol=1e-6, atol=1e-6)
    Yb = oracle.binary_gemm(Wp, alpha, n, Xp, beta, bias=bias)
    assert np.allclose(Yb, ref + bias, rtol=1e-6, atol=1e-6)
    Y0 = g.standard_normal((B, m)).astype(np.float32)
    Ya = oracle.binary_gemm(Wp, alpha, n, Xp, beta, bias=bias, Y=Y0)
    assert np.allclose(Ya, ref + bias + Y0, rtol=1e-6, atol=1e-6)
    # quantization is doing something sensible: more bits -> closer to the dense product
    dense = X.astype(np.float64) @ W.astype(np.float64).T
    rel = np.linalg.norm(ref - dense) / np.linalg.norm(dense)
    assert rel < {1: 0.95, 2: 0.6, 3: 0.35, 4: 0.2}[min(k_w, k_a)]


def sigmoid(a):
    return 1.0 / (1.0 + np.exp(-a))


def setup_cell(g, gates, I, H, B, k_w, k_a):
    Wx = (g.standard_normal((gates * H, I)) * 0.08).astype(np.float32)
    Wh = (g.standard_normal((gates * H, H)) * 0.08).astype(np.float32)
    x = g.standard_normal((B, I)).astype(np.float32)
    h = np.tanh(g.standard_normal((B, H))).astype(np.float32)
    c = g.standard_normal((B, H)).astype(np.float32)
    Wxp, ax = oracle.quantize_rows(Wx, k_w, 2)
    Whp, ah = oracle.quantize_rows(Wh, k_w, 2)
    xq = dequant(*oracle.quantize_rows(x, k_a, 2), I)
    hq = dequant(*oracle.quantize_rows(h, k_a, 2), H)
    Wxq = dequant(Wxp, ax, I)
    Whq = dequant(Whp, ah, H)
    return Wxp, ax, Whp, ah, x, h, c, xq, hq, Wxq, Whq


@pytest.mark.parametrize("k_w,k_a,I,H,B", [(2, 2, 40, 24, 3), (3, 3, 130, 33, 2), (2, 3, 64, 64, 1)])
def test_lstm_step_equals_textbook_cell_on_dequantized(k_w, k_a, I, H, B):
    g = np.random.default_rng(3)
    Wxp, ax, Whp, ah, x, h, c, xq, hq, Wxq, Whq = setup_cell(g, 4, I, H, B, k_w, k_a)
    bias = (g.standard_normal(4 * H) * 0.2).astype(np.float32)
    for b_ in (None, bias):
        a = xq @ Wxq.T + hq @ Whq.T + (0 if b_ is None else b_.astype(np.float64))
        i, f, o = sigmoid(a[:, :H]), sigmoid(a[:, H:2 * H]), sigmoid(a[:, 2 * H:3 * H])
        gg = np.tanh(a[:, 3 * H:])
        c_ref = f * c + i * gg
        h_ref = o * np.tanh(c_ref)
        h_o, c_o = oracle.lstm_step(Wxp, ax, Whp, ah, I, H, b_, x, h, c, k_a, 2)
        assert np.allclose(c_o, c_ref, rtol=1e-6, atol=1e-6)
        assert np.allclose(h_o, h_ref, rtol=1e-6, atol=1e-6)


@pytest.mark.parametrize("k_w,k_a,I,H,B", [(2, 2, 40, 24, 3), (3, 3, 130, 33, 2)])
def test_gru_step_equals_textbook_cell_on_dequantized(k_w, k_a, I, H, B):
    g = np.random.default_rng(4)
    Wxp, ax, Whp, ah, x, h, c, xq, hq, Wxq, Whq = setup_cell(g, 3, I, H, B, k_w, k_a)
    bx = (g.standard_normal(3 * H) * 0.2).astype(np.float32)
    bh = (g.standard_normal(3 * H) * 0.2).astype(np.float32)
    for b1, b2 in ((None, None), (bx, bh)):
        gx = xq @ Wxq.T + (0 if b1 is None else b1.astype(np.float64))
        gh = hq @ Whq.T + (0 if b2 is None else b2.astype(np.float64))
        r = sigmoid(gx[:, :H] + gh[:, :H])
        z = sigmoid(gx[:, H:2 * H] + gh[:, H:2 * H])
        nn = np.tanh(gx[:, 2 * H:] + r * gh[:, 2 * H:])
        h_ref = (1 - z) * nn + z * h
        h_o = oracle.gru_step(Wxp, ax, Whp, ah, I, H, b1, b2, x, h, k_a, 2)
        assert np.allclose(h_o, h_ref, rtol=1e-6, atol=1e-6)


def test_lstm_approaches_unquantized_cell_with_more_bits():
    g = np.random.default_rng(5)
    I = H = 256
    B = 2
    Wx = (g.standard_normal((4 * H, I)) * 0.05).astype(np.float32)
    Wh = (g.standard_normal((4 * H, H)) * 0.05).astype(np.float32)
    x = g.standard_normal((B, I)).astype(np.float32)
    h = np.tanh(g.standard_normal((B, H))).astype(np.float32)
    c = g.standard_normal((B, H)).astype(np.float32)
    a = x.astype(np.float64) @ Wx.T + h.astype(np.float64) @ Wh.T
    c_ref = sigmoid(a[:, H:2 * H]) * c + sigmoid(a[:, :H]) * np.tanh(a[:, 3 * H:])
    h_ref = sigmoid(a[:, 2 * H:3 * H]) * np.tanh(c_ref)
    errs = []
    for k in (1, 2, 3, 4):
        Wxp, ax = oracle.quantize_rows(Wx, k, 2)
        Whp, ah = oracle.quantize_rows(Wh, k, 2)
        h_o, _ = oracle.lstm_step(Wxp, ax, Whp, ah, I, H, None, x, h, c, k, 2)
        errs.append(np.abs(h_o - h_ref).mean())
    assert errs[0] > errs[1] > errs[2] > errs[3]
    assert errs[3] < 0.25 * errs[0]


def test_zero_state_first_step():
    # h_0 = 0: its coefficients are 0, so the hidden-side product vanishes exactly.
    g = np.random.default_rng(6)
    I, H, B = 48, 32, 2
    Wxp, ax, Whp, ah, x, h, c, xq, hq, Wxq, Whq = setup_cell(g, 4, I, H, B, 2, 2)
    z = np.zeros((B, H), np.float32)
    h_o, c_o = oracle.lstm_step(Wxp, ax, Whp, ah, I, H, None, x, z, z, 2, 2)
    a = xq @ Wxq.T
    c_ref = sigmoid(a[:, :H]) * np.tanh(a[:, 3 * H:])
    assert np.allclose(c_o, c_ref, rtol=1e-6, atol=1e-6)
    assert np.allclose(h_o, sigmoid(a[:, 2 * H:3 * H]) * np.tanh(c_ref), rtol=1e-6, atol=1e-6)


def test_threads_do_not_change_results():
    g = np.random.default_rng(7)
    W = g.standard_normal((64, 200)).astype(np.float32)
    oracle.set_threads(1)
    p1, a1 = oracle.quantize_rows(W, 3, 2)
    oracle.set_threads(4)
    p4, a4 = oracle.quantize_rows(W, 3, 2)
    oracle.set_threads(1)
    assert np.array_equal(p1, p4) and np.array_equal(a1, a4)


def _dq(planes, alpha, n):
    k, rows, w = planes.shape
    bits = np.unpackbits(planes.view(np.uint8).reshape(k, rows, w * 4), axis=-1, bitorder="little")[..., :n]
    return np.einsum("krn,rk->rn", bits.astype(np.float64) * 2 - 1, alpha.astype(np.float64))


def test_gru_reset_before_matches_dense_cell_on_dequantized_operands():
    g = np.random.default_rng(31)
    I, H, B, k = 40, 24, 3, 2
    Wx = (g.standard_normal((3 * H, I)) * 0.2).astype(np.float32)
    Wh = (g.standard_normal((3 * H, H)) * 0.2).astype(np.float32)
    bx = (g.standard_normal(3 * H) * 0.1).astype(np.float32)
    bh = (g.standard_normal(3 * H) * 0.1).astype(np.float32)
    x = g.standard_normal((B, I)).astype(np.float32)
    h0 = np.tanh(g.standard_normal((B, H))).astype(np.float32)
    Wxp, ax = oracle.quantize_rows(Wx, k, 2)
    Whp, ah = oracle.quantize_rows(Wh, k, 2)
    h1 = oracle.gru_step_reset_before(Wxp, ax, Whp, ah, I, H, bx, bh, x, h0, k, 2)
    Wxd, Whd = _dq(Wxp, ax, I), _dq(Whp, ah, H)
    q = lambda v: _dq(*oracle.quantize_rows(v, k, 2), v.shape[1])
    sig = lambda t: 1.0 / (1.0 + np.exp(-t))
    a_x = q(x) @ Wxd.T + bx
    a_h = q(h0) @ Whd.T + bh
    r = sig(a_x[:, :H] + a_h[:, :H])
    z = sig(a_x[:, H:2 * H] + a_h[:, H:2 * H])
    gvec = (r * h0).astype(np.float32)
    a_g = q(gvec) @ Whd.T + bh
    n = np.tanh(a_x[:, 2 * H:] + a_g[:, 2 * H:])
    ref = (1 - z) * n + z * h0
    assert np.allclose(h1, ref, rtol=1e-6, atol=1e-6)
    # it is not the reset-after cell in general ...
    h_after = oracle.gru_step(Wxp, ax, Whp, ah, I, H, bx, bh, x, h0, k, 2)
    assert np.abs(h1 - h_after).max() > 1e-3
    # ... but coincides with it when the reset gate is saturated at 1 (r * h = h exactly, and with
    # zero hidden-side bias on the candidate rows r * (U h) = U h)
    bx2, bh2 = bx.copy(), bh.copy()
    bx2[:H] = 60.0
    bh2[2 * H:] = 0.0
    a = oracle.gru_step_reset_before(Wxp, ax, Whp, ah, I, H, bx2, bh2, x, h0, k, 2)
    b = oracle.gru_step(Wxp, ax, Whp, ah, I, H, bx2, bh2, x, h0, k, 2)
    assert np.allclose(a, b, rtol=0, atol=1e-7)
