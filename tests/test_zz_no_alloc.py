"""GPU parity of amq_lstm_step_static (the LSTM step on the library's static scratch, for callers that
cannot allocate) against amq_lstm_step on a caller's workspace, through the C ABI: two calls in a row,
the second with a smaller input, each also checked against the CPU oracle."""
import ctypes as C

import numpy as np
import pytest

import oracle
from gpu_util import assert_vec_close, host, to_dev

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


def _case(L, torch, I, H, B, k_w, k_a, seed):
    g = np.random.default_rng(seed)
    Wx = (g.standard_normal((4 * H, I)) * 0.08).astype(np.float32)
    Wh = (g.standard_normal((4 * H, H)) * 0.08).astype(np.float32)
    bias = (g.standard_normal(4 * H) * 0.1).astype(np.float32)
    x = g.standard_normal((B, I)).astype(np.float32)
    h = np.tanh(g.standard_normal((B, H))).astype(np.float32)
    c = g.standard_normal((B, H)).astype(np.float32)
    Wxp, ax = oracle.quantize_rows(Wx, k_w, 2)
    Whp, ah = oracle.quantize_rows(Wh, k_w, 2)
    d = [to_dev(t) for t in (Wxp, ax, Whp, ah, bias, x, h, c)]
    p = [t.data_ptr() for t in d]
    s = torch.cuda.current_stream().cuda_stream
    need = L.amq_lstm_workspace_bytes(I, H, B, k_a)
    ws = torch.empty(need, dtype=torch.uint8, device=d[0].device)
    h_ws, c_ws = torch.empty_like(d[6]), torch.empty_like(d[7])
    h_st, c_st = torch.full_like(d[6], float("nan")), torch.full_like(d[7], float("nan"))
    say("static-scratch lstm step I=%d H=%d B=%d W%d/A%d (workspace %d bytes)" % (I, H, B, k_w, k_a, need))
    st = L.amq_lstm_step(p[0], p[1], p[2], p[3], I, H, k_w, p[4], p[5], p[6], p[7], B, k_a, 2, h_ws.data_ptr(),
                         c_ws.data_ptr(), ws.data_ptr(), need, s)
    assert st == 0, st
    st = L.amq_lstm_step_static(p[0], p[1], p[2], p[3], I, H, k_w, p[4], p[5], p[6], p[7], B, k_a, 2,
                                h_st.data_ptr(), c_st.data_ptr(), s)
    assert st == 0, st
    torch.cuda.synchronize()
    # same kernels on the same operands: the two entry points agree to the last bit
    assert np.array_equal(host(h_st), host(h_ws)) and np.array_equal(host(c_st), host(c_ws))
    h_ref, c_ref = oracle.lstm_step(Wxp, ax, Whp, ah, I, H, bias, x, h, c, k_a, 2)
    assert_vec_close(host(h_st), h_ref, "h (static scratch)")
    assert_vec_close(host(c_st), c_ref, "c (static scratch)")


def test_static_scratch_lstm_step_two_calls_second_smaller():
    import torch
    import paper_1802_00150_amd as amq
    L = amq.binding.lib()
    oracle.set_threads(oracle.host_threads())
    try:
        # a batch that takes the matrix-core kernel, then a smaller one on the popcount kernel: the
        # second call finds the first call's contents in the scratch
        _case(L, torch, 1024, 512, 40, 3, 3, 11)
        _case(L, torch, 130, 33, 2, 2, 2, 12)
        # a shape that needs the unfused path (pre-activations in the scratch), then a tiny one
        _case(L, torch, 9000, 40, 3, 2, 2, 13)
        _case(L, torch, 17, 5, 1, 1, 1, 14)
    finally:
        oracle.set_threads(1)


def test_static_scratch_rejects_what_does_not_fit():
    import paper_1802_00150_amd as amq
    L = amq.binding.lib()
    p = C.c_void_p(0x10000)
    assert L.amq_lstm_workspace_bytes(1024, 1024, 512, 3) > amq.binding.STATIC_SCRATCH_BYTES
    assert L.amq_lstm_step_static(p, p, p, p, 1024, 1024, 3, None, p, p, p, 512, 3, 2, p, p, None) == 2
    assert L.amq_lstm_step_static(p, p, p, p, 8, 8, 2, None, p, p, None, 1, 2, 2, p, p, None) == 1
