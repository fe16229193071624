"""GPU parity: binary dots (bit-exact), quantized GEMV / GEMM and the grouped GEMV against the
CPU oracle, through the C ABI."""
import numpy as np
import pytest

import oracle
from gpu_util import assert_vec_close, host, to_dev

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


@pytest.fixture(scope="module")
def amq():
    import paper_1802_00150_amd as m
    m.binding.lib()
    return m


def rand_planes(g, k, rows, n):
    wpr = oracle.wpr(n)
    bits = np.zeros((k, rows, wpr * 32), np.uint8)
    bits[:, :, :n] = g.random((k, rows, n)) < 0.5
    return np.packbits(bits, axis=2, bitorder="little").view("<u4").reshape(k, rows, wpr).astype(np.uint32)


SHAPES = [(1, 1), (7, 31), (33, 300), (1200, 300), (130, 600), (257, 1024), (64, 2053), (19, 9000),
          (5, 40000)]


@pytest.mark.parametrize("k_w,k_a", [(1, 1), (2, 2), (2, 3), (3, 3), (4, 4), (3, 1)])
def test_binary_dots_bit_exact(amq, k_w, k_a):
    g = np.random.default_rng(10 * k_w + k_a)
    for (m, n) in SHAPES:
        for batch in (1, 3, 9, 17, 35):
            say("dots kw=%d ka=%d m=%d n=%d B=%d" % (k_w, k_a, m, n, batch))
            Wp = rand_planes(g, k_w, m, n)
            Xp = rand_planes(g, k_a, batch, n)
            ref = oracle.binary_dots(Wp, n, Xp)
            got = host(amq.binary_dots(to_dev(Wp), n, to_dev(Xp)))
            assert np.array_equal(got, ref)


@pytest.mark.parametrize("k_w,k_a", [(1, 1), (2, 2), (2, 3), (3, 3), (4, 4)])
def test_gemm_and_gemv(amq, k_w, k_a):
    g = np.random.default_rng(50 + 10 * k_w + k_a)
    for (m, n) in [(37, 300), (1200, 300), (4096, 1024), (515, 2048), (3000, 1024), (70, 2500)]:
        for batch in (1, 4, 8, 11, 20, 37):
            say("gemm kw=%d ka=%d m=%d n=%d B=%d" % (k_w, k_a, m, n, batch))
            W = (g.standard_normal((m, n)) * 0.02).astype(np.float32)
            X = g.standard_normal((batch, n)).astype(np.float32)
            bias = (g.standard_normal(m) * 0.1).astype(np.float32)
            Wp, alpha = oracle.quantize_rows(W, k_w, 2)
            Xp, beta = oracle.quantize_rows(X, k_a, 2)
            dW, dA, dX, dB, dbias = to_dev(Wp), to_dev(alpha), to_dev(Xp), to_dev(beta), to_dev(bias)
            ref = oracle.binary_gemm(Wp, alpha, n, Xp, beta)
            assert_vec_close(host(amq.binary_gemm(dW, dA, n, dX, dB)), ref)
            refb = oracle.binary_gemm(Wp, alpha, n, Xp, beta, bias=bias)
            assert_vec_close(host(amq.binary_gemm(dW, dA, n, dX, dB, bias=dbias)), refb)
            Y0 = g.standard_normal((batch, m)).astype(np.float32)
            refa = oracle.binary_gemm(Wp, alpha, n, Xp, beta, bias=bias, Y=Y0)
            assert_vec_close(host(amq.binary_gemm(dW, dA, n, dX, dB, bias=dbias, Y=to_dev(Y0))), refa)
            if batch == 1:
                assert_vec_close(host(amq.binary_gemv(dW, dA, n, dX, dB, bias=dbias)), refb)
                assert_vec_close(host(amq.binary_gemv(dW, dA, n, dX, dB, bias=dbias, Y=to_dev(Y0))), refa)


@pytest.mark.parametrize("k_w,k_a,m,n,batch", [
    (2, 2, 10930, 200, 130),    # 9 batch tiles in 3 groups of 3; rows ragged against 16 and against 4
    (2, 3, 8500, 1024, 256),    # the projection's shape class: 4 groups of 4 tiles, last row block partial
    (3, 3, 16404, 256, 100),    # 7 tiles in 4 groups of 2, last group half empty
    (1, 4, 32770, 130, 33),     # one group of 3 tiles, the last with a single entry
    (4, 2, 11000, 1000, 97),    # 7 tiles in 3 groups of 3
])
def test_gemm_many_rows_wide_batch(amq, k_w, k_a, m, n, batch):
    # Plain products with thousands of row blocks and 32 or more columns take the matrix-core kernel
    # that gives each wave several batch tiles; every output is checked, with bias and accumulation.
    g = np.random.default_rng(7000 + 100 * k_w + 10 * k_a + batch)
    say("wide gemm kw=%d ka=%d m=%d n=%d B=%d" % (k_w, k_a, m, n, batch))
    Wp = rand_planes(g, k_w, m, n)
    Xp = rand_planes(g, k_a, batch, n)
    alpha = (np.abs(g.standard_normal((m, k_w))) * 0.02).astype(np.float32)
    beta = np.abs(g.standard_normal((batch, k_a))).astype(np.float32)
    bias = (g.standard_normal(m) * 0.1).astype(np.float32)
    Y0 = g.standard_normal((batch, m)).astype(np.float32)
    dW, dA, dX, dB, dbias = to_dev(Wp), to_dev(alpha), to_dev(Xp), to_dev(beta), to_dev(bias)
    oracle.set_threads(oracle.host_threads())
    ref = oracle.binary_gemm(Wp, alpha, n, Xp, beta)
    refa = oracle.binary_gemm(Wp, alpha, n, Xp, beta, bias=bias, Y=Y0)
    oracle.set_threads(1)
    assert_vec_close(host(amq.binary_gemm(dW, dA, n, dX, dB)), ref)
    assert_vec_close(host(amq.binary_gemm(dW, dA, n, dX, dB, bias=dbias, Y=to_dev(Y0))), refa)


@pytest.mark.parametrize("k_w,k_a,m,batch", [(2, 2, 42000, 1024), (3, 3, 16384, 1024), (2, 3, 10000, 4096)])
def test_gemm_large_batch_shapes_sampled(amq, k_w, k_a, m, batch):
    # The large-batch products bench.py times, in the launch configuration it times them in (the
    # whole product on the GPU); the oracle computes a sample of rows -- the first and last ones, the
    # rows around the boundaries between workgroups' shares, and random ones -- for every batch entry.
    n = 1024
    g = np.random.default_rng(9000 + m + batch)
    say("large-batch gemm kw=%d ka=%d m=%d B=%d" % (k_w, k_a, m, batch))
    Wp = rand_planes(g, k_w, m, n)
    Xp = rand_planes(g, k_a, batch, n)
    alpha = (np.abs(g.standard_normal((m, k_w))) * 0.02).astype(np.float32)
    beta = np.abs(g.standard_normal((batch, k_a))).astype(np.float32)
    bias = (g.standard_normal(m) * 0.1).astype(np.float32)
    Y = host(amq.binary_gemm(to_dev(Wp), to_dev(alpha), n, to_dev(Xp), to_dev(beta), bias=to_dev(bias)))
    rows = np.unique(np.concatenate([np.arange(0, 20), np.arange(m - 20, m),
                                     (np.arange(1, 16) * (m // 16))[:, None].repeat(6, 1).ravel() + np.tile(np.arange(-3, 3), 15),
                                     g.integers(0, m, 40)]))
    oracle.set_threads(oracle.host_threads())
    ref = oracle.binary_gemm(np.ascontiguousarray(Wp[:, rows]), np.ascontiguousarray(alpha[rows]), n, Xp, beta,
                             bias=np.ascontiguousarray(bias[rows]))
    oracle.set_threads(1)
    got = Y[:, rows]
    # per batch entry, the rms over the sampled rows stands for the rms of that entry's output row
    assert_vec_close(got, ref, "sampled rows")


@pytest.mark.parametrize("batch", [1, 8, 64])
@pytest.mark.parametrize("k", [2, 3])
def test_config2_full_pipeline(amq, k, batch):
    # Config 2: quantize W and x on the GPU, multiply on the GPU; the oracle does the same.
    from paper_1802_00150_amd import inputs
    c = inputs.gemv(trial=k, batch=batch)
    say("config2 k=%d B=%d" % (k, batch))
    pW, aW = amq.quantize_weights(to_dev(c["W"]), k, 2)
    pX, bX = amq.quantize_activations(to_dev(c["x"]), k, 2)
    Y = amq.binary_gemm(pW, aW, c["n"], pX, bX)
    oracle.set_threads(oracle.host_threads())
    Wp, alpha = oracle.quantize_rows(c["W"], k, 2)
    Xp, beta = oracle.quantize_rows(c["x"], k, 2)
    oracle.set_threads(1)
    assert np.array_equal(host(pW).view(np.uint32), Wp)
    assert np.array_equal(host(pX).view(np.uint32), Xp)
    assert_vec_close(host(Y), oracle.binary_gemm(Wp, alpha, c["n"], Xp, beta))
    D = host(amq.binary_dots(pW, c["n"], pX))
    assert np.array_equal(D, oracle.binary_dots(Wp, c["n"], Xp))


def test_grouped_gemv(amq):
    g = np.random.default_rng(77)
    G, m, n, k_w, k_a = 5, 700, 1024, 2, 3
    Wp = np.stack([rand_planes(g, k_w, m, n) for _ in range(G)])
    Xp = np.stack([rand_planes(g, k_a, 1, n)[:, 0] for _ in range(G)])          # [G, k_a, wpr]
    alpha = (g.standard_normal((G, m, k_w)) * 0.02).astype(np.float32)
    beta = g.standard_normal((G, k_a)).astype(np.float32)
    bias = g.standard_normal(m).astype(np.float32)
    Y = host(amq.binary_gemv_grouped(to_dev(Wp), to_dev(alpha), n, to_dev(Xp), to_dev(beta), bias=to_dev(bias)))
    for gi in range(G):
        ref = oracle.binary_gemm(Wp[gi], alpha[gi], n, Xp[gi][:, None, :], beta[gi][None, :], bias=bias)
        assert_vec_close(Y[gi][None, :], ref)
