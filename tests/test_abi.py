"""The C-ABI library loads and exports every symbol that include/amq.h declares; host-only
helpers and argument validation work without a GPU (validation precedes any launch)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    from paper_1802_00150_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_1802_00150_amd import build
        build.build()
    return binding.lib()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "amq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(amq_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_are_exported(L):
    names = declared_symbols()
    assert len(names) >= 15
    for name in names:
        assert hasattr(L, name), name
    from paper_1802_00150_amd import binding
    assert sorted(binding.EXPORTS) == names


def test_host_helpers(L):
    assert [L.amq_wpr(n) for n in (1, 128, 129, 300, 1024, 4096)] == [4, 4, 8, 12, 32, 128]
    assert L.amq_wpr(0) == 0
    assert b"gfx950" in L.amq_version()
    assert L.amq_status_string(0) == b"ok"
    assert L.amq_status_string(1) == b"invalid argument"
    assert L.amq_lstm_workspace_bytes(1024, 1024, 64, 3) % 256 == 0
    assert L.amq_lstm_workspace_bytes(1024, 1024, 64, 3) >= 64 * 4096 * 4 + 2 * 3 * 64 * 32 * 4
    assert L.amq_gru_workspace_bytes(1024, 1024, 0, 2) == 0
    L.amq_lstm_sequence_flag_offset.restype = C.c_size_t
    off = L.amq_lstm_sequence_flag_offset(300, 300, 1, 2)
    assert off % 256 == 0 and off + 4 <= L.amq_lstm_workspace_bytes(300, 300, 1, 2)
    assert L.amq_lstm_sequence_flag_offset(300, 300, 8, 2) == C.c_size_t(-1).value


def test_validation_rejects_before_touching_the_device(L):
    # fake (never dereferenced) aligned addresses: validation must fail on the host
    p = C.c_void_p(0x10000)
    null = C.c_void_p(0)
    INVALID, UNSUPPORTED = 1, 2
    assert L.amq_quantize_weights(null, 4, 4, 4, 2, 2, p, p, None) == INVALID
    assert L.amq_quantize_weights(p, 4, 4, 4, 0, 2, p, p, None) == INVALID
    assert L.amq_quantize_weights(p, 4, 4, 4, 5, 2, p, p, None) == INVALID
    assert L.amq_quantize_weights(p, 4, 4, 4, 2, -1, p, p, None) == INVALID
    assert L.amq_quantize_weights(p, 4, 8, 4, 2, 2, p, p, None) == INVALID          # ld < cols
    assert L.amq_quantize_weights(p, 4, 4, 4, 2, 2, C.c_void_p(0x10004), p, None) == INVALID  # misaligned
    assert L.amq_quantize_weights(p, 4, 16385, 16385, 2, 2, p, p, None) == UNSUPPORTED
    assert L.amq_quantize_activations(p, 0, 4, 2, 2, p, p, None) == INVALID
    assert L.amq_binary_dots(p, 4, 4, 2, p, 1, 2, null, None) == INVALID
    assert L.amq_binary_gemm(p, p, 4, 4, 2, p, p, 1, 9, None, 0, p, None) == INVALID
    assert L.amq_binary_gemm(p, p, 4, (1 << 20) + 1, 2, p, p, 1, 2, None, 0, p, None) == UNSUPPORTED
    assert L.amq_binary_gemv_grouped(70000, p, p, 4, 4, 2, p, p, 2, None, p, None) == UNSUPPORTED
    ws = C.c_void_p(0x20000)
    need = L.amq_lstm_workspace_bytes(8, 8, 1, 2)
    assert L.amq_lstm_step(p, p, p, p, 8, 8, 2, None, p, p, p, 1, 2, 2, p, p, ws, need - 1, None) == INVALID
    assert L.amq_lstm_step(p, p, p, p, 8, 8, 2, None, p, p, p, 1, 2, 2, p, p, C.c_void_p(0x20010), need,
                           None) == INVALID
    assert L.amq_lstm_step(p, p, p, p, 8, 8, 2, None, p, p, null, 1, 2, 2, p, p, ws, need, None) == INVALID
    assert L.amq_gru_step(p, p, p, p, 8, 8, 2, None, None, p, p, 1, 2, 2, p, null, 0, None) == INVALID
    assert L.amq_lstm_sequence(p, p, p, p, 8, 8, 2, None, p, 0, p, p, 1, 2, 2, None, ws, need, None) == INVALID
    need_seq = L.amq_lstm_sequence_workspace_bytes(8, 8, 4, 2)
    assert need_seq > L.amq_lstm_workspace_bytes(8, 8, 4, 2) and need_seq % 256 == 0
    assert L.amq_lstm_sequence_workspace_bytes(8, 8, 0, 2) == 0
    half = lambda **kw: L.amq_debug_lstm_split_half(p, p, p, p, 8, 8, 2, None, kw.get("x_next", p), p, kw.get("c", p), 4, 2,
                                                    2, ws, kw.get("bytes", need_seq), kw.get("half", 0), None)
    assert half(half=2) == INVALID
    assert half(x_next=null) == INVALID
    assert half(c=null) == INVALID
    assert half(bytes=need_seq - 1) == INVALID
    need_g = L.amq_gru_workspace_bytes(8, 8, 4, 2)
    assert L.amq_gru_sequence_workspace_bytes(8, 8, 4, 2) > need_g
    assert L.amq_gru_sequence_workspace_bytes(8, 0, 4, 2) == 0
    gseq = lambda **kw: L.amq_gru_sequence(p, p, p, p, 8, 8, 2, None, None, kw.get("xs", p), kw.get("steps", 3),
                                           kw.get("h", p), 4, 2, 2, None, ws, kw.get("bytes", need_g), None)
    assert gseq(steps=0) == INVALID
    assert gseq(xs=null) == INVALID
    assert gseq(h=null) == INVALID
    assert gseq(bytes=need_g - 1) == INVALID
    assert L.amq_lstm_step_packed(p, p, p, p, 8, 8, 2, None, null, p, p, p, p, 1, 2, p, p, None) == INVALID
    assert L.amq_lstm_step_packed(p, p, p, p, 8, 8, 2, None, p, p, p, p, p, 1, 7, p, p, None) == INVALID
    assert L.amq_lstm_step_packed(p, p, p, p, 16385, 16, 2, None, p, p, p, p, p, 4, 2, p, p, None) == UNSUPPORTED
    assert L.amq_lstm_step_packed_grouped(3, p, p, p, p, 8, 8, 2, None, p, p, p, p, null, 2, p, p, None) == INVALID
    assert L.amq_lstm_step_packed_grouped(0, p, p, p, p, 8, 8, 2, None, p, p, p, p, p, 2, p, p, None) == INVALID
    assert L.amq_lstm_step_packed_grouped(70000, p, p, p, p, 8, 8, 2, None, p, p, p, p, p, 2, p, p, None) == UNSUPPORTED
    assert L.amq_lstm_step_packed_grouped(3, p, p, p, p, 9000, 8, 2, None, p, p, p, p, p, 2, p, p, None) == UNSUPPORTED
    assert L.amq_stream_read_probe(p, 24, p, None) == INVALID          # not a multiple of 16
    assert L.amq_stream_read_probe(p, 0, p, None) == INVALID
    assert L.amq_stream_read_probe(null, 32, p, None) == INVALID
    assert L.amq_lstm_step_static(p, p, p, p, 8, 8, 2, None, p, p, null, 1, 2, 2, p, p, None) == INVALID
    # comparison quantizer and error measure
    assert L.amq_quantize_refined_greedy(null, 4, 4, 4, 2, p, p, None) == INVALID
    assert L.amq_quantize_refined_greedy(p, 4, 8, 4, 2, p, p, None) == INVALID
    assert L.amq_quantize_refined_greedy(p, 4, 4, 4, 5, p, p, None) == INVALID
    assert L.amq_quantize_refined_greedy(p, 4, 16385, 16385, 2, p, p, None) == UNSUPPORTED
    assert L.amq_quantize_ternary(null, 4, 4, 4, 2, p, p, None) == INVALID
    assert L.amq_quantize_ternary(p, 4, 8, 4, 2, p, p, None) == INVALID
    assert L.amq_quantize_ternary(p, 4, 4, 4, -1, p, p, None) == INVALID
    assert L.amq_quantize_ternary(p, 4, 16385, 16385, 2, p, p, None) == UNSUPPORTED
    assert L.amq_relative_mse(p, 4, 4, 4, 2, p, p, p, p, null, None) == INVALID
    assert L.amq_relative_mse(p, 0, 4, 4, 2, p, p, p, p, p, None) == INVALID
    assert L.amq_relative_mse(p, 4, 4, 2, 2, p, p, p, p, p, None) == INVALID
    assert L.amq_quantize_weights_ex(p, 4, 4, 4, 2, 2, 4, p, p, None) == INVALID        # unknown flag
    assert L.amq_quantize_weights_ex(null, 4, 4, 4, 2, 2, 1, p, p, None) == INVALID
    assert L.amq_dequantize(p, p, 4, 8, 2, p, 4, None) == INVALID                       # ld_out < cols
    assert L.amq_dequantize(p, null, 4, 8, 2, p, 8, None) == INVALID
    assert L.amq_clip(null, C.c_int64(4), C.c_float(-1.0), C.c_float(1.0), None) == INVALID
    assert L.amq_clip(p, C.c_int64(4), C.c_float(1.0), C.c_float(-1.0), None) == INVALID  # lo > hi
    need_rb = L.amq_gru_reset_before_workspace_bytes(8, 8, 1, 2)
    assert need_rb > L.amq_gru_workspace_bytes(8, 8, 1, 2)
    assert L.amq_gru_step_reset_before(p, p, p, p, 8, 8, 2, None, None, p, p, 1, 2, 2, p, None, ws, need_rb - 1, None) == INVALID
    assert L.amq_gru_step_reset_before(p, p, p, p, 8, 8, 2, None, None, p, null, 1, 2, 2, p, None, ws, need_rb, None) == INVALID
    # language-model entry points
    assert L.amq_embedding_lookup(p, p, 10, 8, 2, null, 1, p, p, None) == INVALID
    assert L.amq_embedding_lookup(p, p, 0, 8, 2, p, 1, p, p, None) == INVALID
    assert L.amq_embedding_lookup(p, p, 10, 8, 5, p, 1, p, p, None) == INVALID
    assert L.amq_embedding_lookup(p, p, 10, 1 << 15, 2, p, 1, p, p, None) == UNSUPPORTED
    assert L.amq_log_softmax(p, 0, 8, p, None) == INVALID
    assert L.amq_log_softmax(null, 1, 8, p, None) == INVALID
    assert L.amq_log_softmax(p, 1, (1 << 31) + 1, p, None) == UNSUPPORTED
    need_s = L.amq_softmax_layer_workspace_bytes(16, 8, 1, 2)
    assert need_s > 0 and need_s % 256 == 0
    assert L.amq_softmax_layer_workspace_bytes(16, 8, 1, 0) == 0
    assert L.amq_softmax_layer(p, p, 16, 8, 2, None, p, 1, 2, 2, p, ws, need_s - 1, None) == INVALID
    assert L.amq_softmax_layer(p, p, 16, 8, 2, None, p, 1, 2, -1, p, ws, need_s, None) == INVALID
    assert L.amq_softmax_layer(p, p, 16, 8, 2, None, null, 1, 2, 2, p, ws, need_s, None) == INVALID
    need_l = L.amq_lm_workspace_bytes(8, 8, 16, 1, 2, 3)
    assert need_l == need + L.amq_softmax_layer_workspace_bytes(16, 8, 1, 3)
    lm = lambda **kw: L.amq_lm_step(p, p, kw.get("vocab", 10), 8, p, p, p, p, 8, 2, None, p, p, 16, kw.get("k_ws", 2),
                                    None, kw.get("ids", p), p, p, 1, 2, kw.get("k_as", 3), 2, p, ws,
                                    kw.get("bytes", need_l), None)
    assert lm(bytes=need_l - 1) == INVALID
    assert lm(ids=null) == INVALID
    assert lm(vocab=0) == INVALID
    assert lm(k_ws=5) == INVALID
    assert lm(k_as=0) == INVALID
    need_q = L.amq_lm_sequence_workspace_bytes(8, 8, 16, 1, 2, 3)
    assert need_q > need_l
    lmq = lambda **kw: L.amq_lm_sequence(p, p, 10, 8, p, p, p, p, 8, 2, None, p, p, 16, 2, None, kw.get("ids", p),
                                         kw.get("steps", 3), p, p, 1, 2, 3, 2, p, ws, kw.get("bytes", need_q), None)
    assert lmq(bytes=need_q - 1) == INVALID
    assert lmq(steps=0) == INVALID
    assert lmq(ids=null) == INVALID
    need_s = L.amq_lm_sequence_score_workspace_bytes(8, 8, 16, 1, 2, 3)
    assert need_s > need_q
    lms = lambda **kw: L.amq_lm_sequence_score(p, p, 10, 8, p, p, p, p, 8, 2, None, p, p, 16, 2, None, p,
                                               kw.get("targets", p), kw.get("steps", 3), p, p, 1, 2, 3, 2,
                                               kw.get("out", p), ws, kw.get("bytes", need_s), None)
    assert lms(bytes=need_s - 1) == INVALID
    assert lms(steps=0) == INVALID
    assert lms(targets=null) == INVALID
    assert lms(out=null) == INVALID
    assert L.amq_lm_sequence_score_workspace_bytes(8, 8, 16, 0, 2, 3) == 0


def test_binding_refuses_cpu_tensors():
    import torch
    import paper_1802_00150_amd as amq
    with pytest.raises(amq.AmqError):
        amq.quantize_activations(torch.zeros(2, 8), 2, 2)
