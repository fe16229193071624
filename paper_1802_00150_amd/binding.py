"""Thin Python binding of the C ABI in include/amq.h.

Argument marshalling only: every function takes torch tensors that already live on the GPU,
passes their device pointers and the current HIP stream to the entry point of the same name,
and raises on a non-zero status.  There is no CPU fallback: without the built library, or on
tensors that are not on a GPU, every call fails loudly.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# AMQ_LIBRARY (read once, at load) names another build of the same library, e.g. the profiling build
# libamq_phases.so with in-kernel phase timers
LIB_PATH = os.environ.get("AMQ_LIBRARY") or os.path.join(_HERE, "libamq.so")

EXPORTS = [
    "amq_wpr", "amq_version", "amq_status_string", "amq_last_hip_error",
    "amq_quantize_weights", "amq_quantize_activations", "amq_ls_update", "amq_bst_assign",
    "amq_binary_dots", "amq_binary_gemv", "amq_binary_gemm", "amq_binary_gemv_grouped",
    "amq_lstm_workspace_bytes", "amq_lstm_step", "amq_lstm_step_static", "amq_lstm_step_packed",
    "amq_lstm_step_packed_grouped", "amq_stream_read_probe", "amq_lstm_sequence",
    "amq_lstm_sequence_flag_offset", "amq_lstm_sequence_workspace_bytes", "amq_debug_set_sequence_spin_limit",
    "amq_gru_sequence", "amq_gru_sequence_workspace_bytes",
    "amq_debug_lstm_split_half",
    "amq_gru_workspace_bytes", "amq_gru_step",
    "amq_embedding_lookup", "amq_log_softmax", "amq_softmax_layer_workspace_bytes", "amq_softmax_layer",
    "amq_lm_workspace_bytes", "amq_lm_step", "amq_lm_sequence_workspace_bytes", "amq_lm_sequence",
    "amq_lm_sequence_score_workspace_bytes", "amq_lm_sequence_score",
    "amq_quantize_refined_greedy", "amq_quantize_ternary", "amq_relative_mse",
    "amq_quantize_weights_ex", "amq_dequantize", "amq_clip",
    "amq_gru_reset_before_workspace_bytes", "amq_gru_step_reset_before",
]

_lib = None
_p, _i64, _int, _sz = C.c_void_p, C.c_int64, C.c_int, C.c_size_t


class AmqError(RuntimeError):
    pass


def lib():
    """Load libamq.so (built by paper_1802_00150_amd/build.py).  Raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise AmqError("libamq.so is not built: run `python -m paper_1802_00150_amd.build` "
                           "(or __graft_entry__.build()) first")
        L = C.CDLL(LIB_PATH)
        L.amq_wpr.argtypes, L.amq_wpr.restype = [_i64], _i64
        L.amq_version.restype = C.c_char_p
        L.amq_status_string.argtypes, L.amq_status_string.restype = [_int], C.c_char_p
        L.amq_last_hip_error.restype = _int
        L.amq_quantize_weights.argtypes = [_p, _i64, _i64, _i64, _int, _int, _p, _p, _p]
        L.amq_quantize_activations.argtypes = [_p, _i64, _i64, _int, _int, _p, _p, _p]
        L.amq_ls_update.argtypes = [_p, _i64, _i64, _int, _p, _p, _p]
        L.amq_bst_assign.argtypes = [_p, _i64, _i64, _int, _p, _p, _p]
        L.amq_binary_dots.argtypes = [_p, _i64, _i64, _int, _p, _i64, _int, _p, _p]
        L.amq_binary_gemv.argtypes = [_p, _p, _i64, _i64, _int, _p, _p, _int, _p, _int, _p, _p]
        L.amq_binary_gemm.argtypes = [_p, _p, _i64, _i64, _int, _p, _p, _i64, _int, _p, _int, _p, _p]
        L.amq_binary_gemv_grouped.argtypes = [_i64, _p, _p, _i64, _i64, _int, _p, _p, _int, _p, _p, _p]
        L.amq_lstm_workspace_bytes.argtypes, L.amq_lstm_workspace_bytes.restype = [_i64, _i64, _i64, _int], _sz
        L.amq_gru_workspace_bytes.argtypes, L.amq_gru_workspace_bytes.restype = [_i64, _i64, _i64, _int], _sz
        L.amq_lstm_sequence_flag_offset.argtypes = [_i64, _i64, _i64, _int]
        L.amq_lstm_sequence_flag_offset.restype = _sz
        L.amq_lstm_sequence_workspace_bytes.argtypes = [_i64, _i64, _i64, _int]
        L.amq_lstm_sequence_workspace_bytes.restype = _sz
        L.amq_gru_sequence_workspace_bytes.argtypes = [_i64, _i64, _i64, _int]
        L.amq_gru_sequence_workspace_bytes.restype = _sz
        L.amq_gru_sequence.argtypes = [_p, _p, _p, _p, _i64, _i64, _int, _p, _p, _p, _i64, _p, _i64, _int, _int, _p,
                                       _p, _sz, _p]
        L.amq_debug_lstm_split_half.argtypes = [_p, _p, _p, _p, _i64, _i64, _int, _p, _p, _p, _p, _i64, _int, _int, _p, _sz,
                                                _int, _p]
        L.amq_debug_set_sequence_spin_limit.argtypes = [C.c_uint]
        L.amq_debug_set_sequence_spin_limit.restype = None
        L.amq_lstm_step.argtypes = [_p, _p, _p, _p, _i64, _i64, _int, _p, _p, _p, _p, _i64, _int, _int, _p, _p,
                                    _p, _sz, _p]
        L.amq_lstm_step_static.argtypes = [_p, _p, _p, _p, _i64, _i64, _int, _p, _p, _p, _p, _i64, _int, _int, _p, _p,
                                           _p]
        L.amq_lstm_step_packed.argtypes = [_p, _p, _p, _p, _i64, _i64, _int, _p, _p, _p, _p, _p, _p, _i64, _int,
                                           _p, _p, _p]
        L.amq_lstm_step_packed_grouped.argtypes = [_i64, _p, _p, _p, _p, _i64, _i64, _int, _p, _p, _p, _p, _p, _p, _int,
                                                   _p, _p, _p]
        L.amq_stream_read_probe.argtypes = [_p, _sz, _p, _p]
        L.amq_lstm_sequence.argtypes = [_p, _p, _p, _p, _i64, _i64, _int, _p, _p, _i64, _p, _p, _i64, _int,
                                        _int, _p, _p, _sz, _p]
        L.amq_gru_step.argtypes = [_p, _p, _p, _p, _i64, _i64, _int, _p, _p, _p, _p, _i64, _int, _int, _p, _p,
                                   _sz, _p]
        L.amq_embedding_lookup.argtypes = [_p, _p, _i64, _i64, _int, _p, _i64, _p, _p, _p]
        L.amq_log_softmax.argtypes = [_p, _i64, _i64, _p, _p]
        L.amq_softmax_layer_workspace_bytes.argtypes = [_i64, _i64, _i64, _int]
        L.amq_softmax_layer_workspace_bytes.restype = _sz
        L.amq_softmax_layer.argtypes = [_p, _p, _i64, _i64, _int, _p, _p, _i64, _int, _int, _p, _p, _sz, _p]
        L.amq_lm_workspace_bytes.argtypes, L.amq_lm_workspace_bytes.restype = [_i64, _i64, _i64, _i64, _int, _int], _sz
        L.amq_lm_step.argtypes = [_p, _p, _i64, _i64, _p, _p, _p, _p, _i64, _int, _p, _p, _p, _i64, _int, _p,
                                  _p, _p, _p, _i64, _int, _int, _int, _p, _p, _sz, _p]
        L.amq_lm_sequence_workspace_bytes.argtypes = [_i64, _i64, _i64, _i64, _int, _int]
        L.amq_lm_sequence_workspace_bytes.restype = _sz
        L.amq_lm_sequence_score_workspace_bytes.argtypes = [_i64, _i64, _i64, _i64, _int, _int]
        L.amq_lm_sequence_score_workspace_bytes.restype = _sz
        L.amq_lm_sequence_score.argtypes = [_p, _p, _i64, _i64, _p, _p, _p, _p, _i64, _int, _p, _p, _p, _i64, _int, _p,
                                            _p, _p, _i64, _p, _p, _i64, _int, _int, _int, _p, _p, _sz, _p]
        L.amq_lm_sequence.argtypes = [_p, _p, _i64, _i64, _p, _p, _p, _p, _i64, _int, _p, _p, _p, _i64, _int, _p,
                                      _p, _i64, _p, _p, _i64, _int, _int, _int, _p, _p, _sz, _p]
        L.amq_quantize_refined_greedy.argtypes = [_p, _i64, _i64, _i64, _int, _p, _p, _p]
        L.amq_quantize_ternary.argtypes = [_p, _i64, _i64, _i64, _int, _p, _p, _p]
        L.amq_relative_mse.argtypes = [_p, _i64, _i64, _i64, _int, _p, _p, _p, _p, _p, _p]
        L.amq_gru_reset_before_workspace_bytes.argtypes = [_i64, _i64, _i64, _int]
        L.amq_gru_reset_before_workspace_bytes.restype = _sz
        L.amq_gru_step_reset_before.argtypes = [_p, _p, _p, _p, _i64, _i64, _int, _p, _p, _p, _p, _i64, _int, _int, _p, _p,
                                                _p, _sz, _p]
        L.amq_quantize_weights_ex.argtypes = [_p, _i64, _i64, _i64, _int, _int, _int, _p, _p, _p]
        L.amq_dequantize.argtypes = [_p, _p, _i64, _i64, _int, _p, _i64, _p]
        L.amq_clip.argtypes = [_p, _i64, C.c_float, C.c_float, _p]
        _lib = L
    return _lib


def _check(status):
    if status != 0:
        L = lib()
        msg = L.amq_status_string(status).decode()
        if status == 3:
            msg += " (hipError %d)" % L.amq_last_hip_error()
        raise AmqError(msg)


def _dev(t, dtype):
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise AmqError("expected a GPU tensor")
    if t.dtype != dtype or not t.is_contiguous():
        raise AmqError("expected a contiguous %s tensor, got %s" % (dtype, t.dtype))
    return t.data_ptr()


def _opt(t):
    return None if t is None else _dev(t, torch.float32)


def _stream():
    return torch.cuda.current_stream().cuda_stream


def wpr(n):
    return int(lib().amq_wpr(int(n)))


def version():
    return lib().amq_version().decode()


def _empty(shape, dtype, like):
    return torch.empty(shape, dtype=dtype, device=like.device)


QUANT_FINAL_LS = 1


def quantize_weights(W, k, T, final_ls=False):
    """W [rows, cols] float32 (rows may be strided) -> planes [k, rows, wpr] int32, alpha [rows, k].
    final_ls: one more coefficient update (Eq. 5) after the last code assignment."""
    if W.dim() != 2 or W.stride(1) != 1 or W.dtype != torch.float32 or not W.is_cuda:
        raise AmqError("expected a 2-D float32 GPU tensor with unit column stride")
    rows, cols = W.shape
    planes = _empty((k, rows, wpr(cols)), torch.int32, W)
    alpha = _empty((rows, k), torch.float32, W)
    if final_ls:
        _check(lib().amq_quantize_weights_ex(W.data_ptr(), rows, cols, W.stride(0), k, T, QUANT_FINAL_LS,
                                             planes.data_ptr(), alpha.data_ptr(), _stream()))
    else:
        _check(lib().amq_quantize_weights(W.data_ptr(), rows, cols, W.stride(0), k, T, planes.data_ptr(),
                                          alpha.data_ptr(), _stream()))
    return planes, alpha


def quantize_activations(X, k, T):
    """X [batch, n] float32 -> planes [k, batch, wpr] int32, beta [batch, k]."""
    batch, n = X.shape
    planes = _empty((k, batch, wpr(n)), torch.int32, X)
    beta = _empty((batch, k), torch.float32, X)
    _check(lib().amq_quantize_activations(_dev(X, torch.float32), batch, n, k, T, planes.data_ptr(),
                                          beta.data_ptr(), _stream()))
    return planes, beta


def ls_update(X, planes, coef):
    """Eq. 5 with the codes given; returns the updated copy of coef."""
    rows, n = X.shape
    k = planes.shape[0]
    out = coef.clone()
    _check(lib().amq_ls_update(_dev(X, torch.float32), rows, n, k, _dev(planes, torch.int32),
                               _dev(out, torch.float32), _stream()))
    return out


def bst_assign(X, coef):
    """Alg. 1 with the coefficients given; returns planes [k, rows, wpr]."""
    rows, n = X.shape
    k = coef.shape[1]
    planes = _empty((k, rows, wpr(n)), torch.int32, X)
    _check(lib().amq_bst_assign(_dev(X, torch.float32), rows, n, k, _dev(coef, torch.float32),
                                planes.data_ptr(), _stream()))
    return planes


def binary_dots(Wp, n, Xp):
    k_w, m, _ = Wp.shape
    k_a, batch, _ = Xp.shape
    D = _empty((batch, m, k_w, k_a), torch.int32, Wp)
    _check(lib().amq_binary_dots(_dev(Wp, torch.int32), m, n, k_w, _dev(Xp, torch.int32), batch, k_a,
                                 D.data_ptr(), _stream()))
    return D


def binary_gemm(Wp, alpha, n, Xp, beta, bias=None, Y=None):
    """Y [batch, m]; if Y is given the product is accumulated into it (in place)."""
    k_w, m, _ = Wp.shape
    k_a, batch, _ = Xp.shape
    acc = Y is not None
    if not acc:
        Y = _empty((batch, m), torch.float32, Wp)
    _check(lib().amq_binary_gemm(_dev(Wp, torch.int32), _dev(alpha, torch.float32), m, n, k_w,
                                 _dev(Xp, torch.int32), _dev(beta, torch.float32), batch, k_a, _opt(bias),
                                 1 if acc else 0, _dev(Y, torch.float32), _stream()))
    return Y


def binary_gemv(Wp, alpha, n, Xp, beta, bias=None, Y=None):
    k_w, m, _ = Wp.shape
    k_a = Xp.shape[0]
    acc = Y is not None
    if not acc:
        Y = _empty((1, m), torch.float32, Wp)
    _check(lib().amq_binary_gemv(_dev(Wp, torch.int32), _dev(alpha, torch.float32), m, n, k_w,
                                 _dev(Xp, torch.int32), _dev(beta, torch.float32), k_a, _opt(bias),
                                 1 if acc else 0, _dev(Y, torch.float32), _stream()))
    return Y


def binary_gemv_grouped(Wp, alpha, n, Xp, beta, bias=None, Y=None):
    """Wp [G, k_w, m, wpr], alpha [G, m, k_w], Xp [G, k_a, wpr], beta [G, k_a] -> Y [G, m]."""
    G, k_w, m, _ = Wp.shape
    k_a = Xp.shape[1]
    if Y is None:
        Y = _empty((G, m), torch.float32, Wp)
    _check(lib().amq_binary_gemv_grouped(G, _dev(Wp, torch.int32), _dev(alpha, torch.float32), m, n, k_w,
                                         _dev(Xp, torch.int32), _dev(beta, torch.float32), k_a, _opt(bias),
                                         _dev(Y, torch.float32), _stream()))
    return Y


def lstm_workspace(I, H, B, k_a, device):
    nbytes = int(lib().amq_lstm_workspace_bytes(I, H, B, k_a))
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def lstm_sequence_workspace(I, H, B, k_a, device):
    """Workspace with which lstm_sequence takes the input products off the recurrent chain (B > 1)."""
    nbytes = int(lib().amq_lstm_sequence_workspace_bytes(I, H, B, k_a))
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def gru_workspace(I, H, B, k_a, device):
    nbytes = int(lib().amq_gru_workspace_bytes(I, H, B, k_a))
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def lstm_step(Wxp, alpha_x, Whp, alpha_h, I, H, bias, x, h_prev, c_prev, k_a, T, ws=None, h_out=None,
              c_out=None):
    k_w = Wxp.shape[0]
    B = x.shape[0]
    if ws is None:
        ws = lstm_workspace(I, H, B, k_a, x.device)
    if h_out is None:
        h_out = torch.empty_like(h_prev)
    if c_out is None:
        c_out = torch.empty_like(c_prev)
    _check(lib().amq_lstm_step(_dev(Wxp, torch.int32), _dev(alpha_x, torch.float32), _dev(Whp, torch.int32),
                               _dev(alpha_h, torch.float32), I, H, k_w, _opt(bias), _dev(x, torch.float32),
                               _dev(h_prev, torch.float32), _dev(c_prev, torch.float32), B, k_a, T,
                               _dev(h_out, torch.float32), _dev(c_out, torch.float32), ws.data_ptr(),
                               ws.numel(), _stream()))
    return h_out, c_out


STATIC_SCRATCH_BYTES = 4 << 20


def lstm_step_static(Wxp, alpha_x, Whp, alpha_h, I, H, bias, x, h_prev, c_prev, k_a, T, h_out, c_out):
    """lstm_step on the library's static scratch: the call allocates nothing, so the outputs are
    arguments too."""
    _check(lib().amq_lstm_step_static(_dev(Wxp, torch.int32), _dev(alpha_x, torch.float32),
                                      _dev(Whp, torch.int32), _dev(alpha_h, torch.float32), I, H, Wxp.shape[0],
                                      _opt(bias), _dev(x, torch.float32), _dev(h_prev, torch.float32),
                                      _dev(c_prev, torch.float32), x.shape[0], k_a, T,
                                      _dev(h_out, torch.float32), _dev(c_out, torch.float32), _stream()))
    return h_out, c_out


def lstm_step_packed(Wxp, alpha_x, Whp, alpha_h, I, H, bias, Xp, beta_x, Hp, beta_h, c_prev, h_out=None,
                     c_out=None):
    """LSTM step on operands that are already quantized (Xp [k_a, B, wpr(I)], Hp [k_a, B, wpr(H)])."""
    k_w = Wxp.shape[0]
    k_a, B, _ = Xp.shape
    if h_out is None:
        h_out = torch.empty_like(c_prev)
    if c_out is None:
        c_out = torch.empty_like(c_prev)
    _check(lib().amq_lstm_step_packed(_dev(Wxp, torch.int32), _dev(alpha_x, torch.float32),
                                      _dev(Whp, torch.int32), _dev(alpha_h, torch.float32), I, H, k_w,
                                      _opt(bias), _dev(Xp, torch.int32), _dev(beta_x, torch.float32),
                                      _dev(Hp, torch.int32), _dev(beta_h, torch.float32),
                                      _dev(c_prev, torch.float32), B, k_a, _dev(h_out, torch.float32),
                                      _dev(c_out, torch.float32), _stream()))
    return h_out, c_out


def lstm_step_packed_grouped(Wxp, alpha_x, Whp, alpha_h, I, H, bias, Xp, beta_x, Hp, beta_h, c_prev, h_out=None,
                             c_out=None):
    """G independent batch-1 LSTM steps: Wxp [G, k_w, 4H, wpr(I)], alpha_x [G, 4H, k_w], Whp, alpha_h likewise,
    Xp [G, k_a, wpr(I)], beta_x [G, k_a], Hp, beta_h likewise, c_prev [G, H] -> h_out, c_out [G, H]."""
    G, k_w = Wxp.shape[0], Wxp.shape[1]
    k_a = Xp.shape[1]
    if h_out is None:
        h_out = torch.empty_like(c_prev)
    if c_out is None:
        c_out = torch.empty_like(c_prev)
    _check(lib().amq_lstm_step_packed_grouped(G, _dev(Wxp, torch.int32), _dev(alpha_x, torch.float32),
                                              _dev(Whp, torch.int32), _dev(alpha_h, torch.float32), I, H, k_w,
                                              _opt(bias), _dev(Xp, torch.int32), _dev(beta_x, torch.float32),
                                              _dev(Hp, torch.int32), _dev(beta_h, torch.float32),
                                              _dev(c_prev, torch.float32), k_a, _dev(h_out, torch.float32),
                                              _dev(c_out, torch.float32), _stream()))
    return h_out, c_out


STREAM_PROBE_SINK_WORDS = 4096


def stream_read_probe(buf, sink=None):
    """Reads the whole tensor `buf` (bytes a multiple of 16) once; returns the per-workgroup checksums."""
    if sink is None:
        sink = torch.empty(STREAM_PROBE_SINK_WORDS, dtype=torch.int64, device=buf.device)
    if not buf.is_cuda or not buf.is_contiguous():
        raise AmqError("expected a contiguous GPU tensor")
    _check(lib().amq_stream_read_probe(buf.data_ptr(), buf.numel() * buf.element_size(), sink.data_ptr(), _stream()))
    return sink


def lstm_sequence(Wxp, alpha_x, Whp, alpha_h, I, H, bias, xs, h, c, k_a, T, ws=None, hs=None):
    """xs [steps, B, I]; h, c [B, H] are updated in place; hs [steps, B, H] optional."""
    k_w = Wxp.shape[0]
    steps, B, _ = xs.shape
    if ws is None:
        ws = lstm_sequence_workspace(I, H, B, k_a, xs.device)
    _check(lib().amq_lstm_sequence(_dev(Wxp, torch.int32), _dev(alpha_x, torch.float32),
                                   _dev(Whp, torch.int32), _dev(alpha_h, torch.float32), I, H, k_w,
                                   _opt(bias), _dev(xs, torch.float32), steps, _dev(h, torch.float32),
                                   _dev(c, torch.float32), B, k_a, T,
                                   None if hs is None else _dev(hs, torch.float32), ws.data_ptr(),
                                   ws.numel(), _stream()))
    return h, c


def gru_step_reset_before(Wxp, alpha_x, Whp, alpha_h, I, H, bias_x, bias_h, x, h_prev, k_a, T, ws=None, h_out=None,
                          g_out=None):
    """GRU step with the reset gate applied to the previous state before the candidate's product.
    g_out [B, H] (optional) receives r * h_prev."""
    k_w = Wxp.shape[0]
    B = x.shape[0]
    if ws is None:
        ws = torch.empty(int(lib().amq_gru_reset_before_workspace_bytes(I, H, B, k_a)), dtype=torch.uint8,
                         device=x.device)
    if h_out is None:
        h_out = torch.empty_like(h_prev)
    _check(lib().amq_gru_step_reset_before(_dev(Wxp, torch.int32), _dev(alpha_x, torch.float32),
                                           _dev(Whp, torch.int32), _dev(alpha_h, torch.float32), I, H, k_w,
                                           _opt(bias_x), _opt(bias_h), _dev(x, torch.float32),
                                           _dev(h_prev, torch.float32), B, k_a, T, _dev(h_out, torch.float32),
                                           _opt(g_out), ws.data_ptr(), ws.numel(), _stream()))
    return h_out


def debug_set_sequence_spin_limit(polls):
    """Test hook: polls before a wait of the one-launch recurrence gives up (0 restores the default)."""
    lib().amq_debug_set_sequence_spin_limit(int(polls))


def lstm_sequence_abandoned(ws, I, H, B, k_a):
    """True if the last lstm_sequence call on workspace `ws` gave up a bounded wait (see include/amq.h)."""
    off = int(lib().amq_lstm_sequence_flag_offset(I, H, B, k_a))
    if off == C.c_size_t(-1).value:
        return False
    return bool(ws[off:off + 4].view(torch.int32).item() != 0)


def gru_step(Wxp, alpha_x, Whp, alpha_h, I, H, bias_x, bias_h, x, h_prev, k_a, T, ws=None, h_out=None):
    k_w = Wxp.shape[0]
    B = x.shape[0]
    if ws is None:
        ws = gru_workspace(I, H, B, k_a, x.device)
    if h_out is None:
        h_out = torch.empty_like(h_prev)
    _check(lib().amq_gru_step(_dev(Wxp, torch.int32), _dev(alpha_x, torch.float32), _dev(Whp, torch.int32),
                              _dev(alpha_h, torch.float32), I, H, k_w, _opt(bias_x), _opt(bias_h),
                              _dev(x, torch.float32), _dev(h_prev, torch.float32), B, k_a, T,
                              _dev(h_out, torch.float32), ws.data_ptr(), ws.numel(), _stream()))
    return h_out


def gru_sequence_workspace(I, H, B, k_a, device):
    """Workspace with which gru_sequence takes the input products off the recurrent chain (B > 1)."""
    nbytes = int(lib().amq_gru_sequence_workspace_bytes(I, H, B, k_a))
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def gru_sequence(Wxp, alpha_x, Whp, alpha_h, I, H, bias_x, bias_h, xs, h, k_a, T, ws=None, hs=None):
    """xs [steps, B, I]; h [B, H] is updated in place; hs [steps, B, H] optional."""
    k_w = Wxp.shape[0]
    steps, B, _ = xs.shape
    if ws is None:
        ws = gru_sequence_workspace(I, H, B, k_a, xs.device)
    _check(lib().amq_gru_sequence(_dev(Wxp, torch.int32), _dev(alpha_x, torch.float32), _dev(Whp, torch.int32),
                                  _dev(alpha_h, torch.float32), I, H, k_w, _opt(bias_x), _opt(bias_h),
                                  _dev(xs, torch.float32), steps, _dev(h, torch.float32), B, k_a, T,
                                  None if hs is None else _dev(hs, torch.float32), ws.data_ptr(), ws.numel(),
                                  _stream()))
    return h


def embedding_lookup(Ep, alpha_e, n, ids):
    """Rows ids [B] (int64) of a quantized table Ep [k, vocab, wpr(n)], alpha_e [vocab, k] ->
    Xp [k, B, wpr(n)], beta [B, k]."""
    k, vocab, w = Ep.shape
    B = ids.shape[0]
    Xp = _empty((k, B, w), torch.int32, Ep)
    beta = _empty((B, k), torch.float32, Ep)
    _check(lib().amq_embedding_lookup(_dev(Ep, torch.int32), _dev(alpha_e, torch.float32), vocab, n, k,
                                      _dev(ids, torch.int64), B, Xp.data_ptr(), beta.data_ptr(), _stream()))
    return Xp, beta


def log_softmax(Y, out=None):
    """Row-wise log-softmax of Y [B, V]; out may be Y itself."""
    B, V = Y.shape
    if out is None:
        out = torch.empty_like(Y)
    _check(lib().amq_log_softmax(_dev(Y, torch.float32), B, V, _dev(out, torch.float32), _stream()))
    return out


def softmax_layer_workspace(V, H, B, k_a, device):
    nbytes = int(lib().amq_softmax_layer_workspace_bytes(V, H, B, k_a))
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def softmax_layer(Wsp, alpha_s, H, bias, h, k_a, T, ws=None, logprob=None):
    """log softmax(W_s h + b_s) with W_s quantized (Wsp [k_w, V, wpr(H)]) and h [B, H] quantized on line."""
    k_w, V, _ = Wsp.shape
    B = h.shape[0]
    if ws is None:
        ws = softmax_layer_workspace(V, H, B, k_a, h.device)
    if logprob is None:
        logprob = _empty((B, V), torch.float32, h)
    _check(lib().amq_softmax_layer(_dev(Wsp, torch.int32), _dev(alpha_s, torch.float32), V, H, k_w, _opt(bias),
                                   _dev(h, torch.float32), B, k_a, T, _dev(logprob, torch.float32),
                                   ws.data_ptr(), ws.numel(), _stream()))
    return logprob


def lm_workspace(E, H, V, B, k_a, k_as, device):
    nbytes = int(lib().amq_lm_workspace_bytes(E, H, V, B, k_a, k_as))
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def lm_step(Ep, alpha_e, E, Wxp, alpha_x, Whp, alpha_h, H, bias, Wsp, alpha_s, bias_s, ids, h, c, k_a, k_as, T,
            ws=None, logprob=None):
    """One language-model step: ids [B] -> embedding rows -> LSTM (h, c updated in place) -> log-probabilities
    [B, V]."""
    vocab = Ep.shape[1]
    k_w = Wxp.shape[0]
    k_ws, V, _ = Wsp.shape
    B = ids.shape[0]
    if ws is None:
        ws = lm_workspace(E, H, V, B, k_a, k_as, h.device)
    if logprob is None:
        logprob = _empty((B, V), torch.float32, h)
    _check(lib().amq_lm_step(_dev(Ep, torch.int32), _dev(alpha_e, torch.float32), vocab, E,
                             _dev(Wxp, torch.int32), _dev(alpha_x, torch.float32), _dev(Whp, torch.int32),
                             _dev(alpha_h, torch.float32), H, k_w, _opt(bias), _dev(Wsp, torch.int32),
                             _dev(alpha_s, torch.float32), V, k_ws, _opt(bias_s), _dev(ids, torch.int64),
                             _dev(h, torch.float32), _dev(c, torch.float32), B, k_a, k_as, T,
                             _dev(logprob, torch.float32), ws.data_ptr(), ws.numel(), _stream()))
    return logprob


def lm_sequence(Ep, alpha_e, E, Wxp, alpha_x, Whp, alpha_h, H, bias, Wsp, alpha_s, bias_s, ids, h, c, k_a, k_as, T,
                ws=None, logprob=None):
    """ids [steps, B] -> logprob [steps, B, V]; h, c [B, H] updated in place."""
    vocab = Ep.shape[1]
    k_w = Wxp.shape[0]
    k_ws, V, _ = Wsp.shape
    steps, B = ids.shape
    if ws is None:
        ws = torch.empty(int(lib().amq_lm_sequence_workspace_bytes(E, H, V, B, k_a, k_as)), dtype=torch.uint8,
                         device=h.device)
    if logprob is None:
        logprob = _empty((steps, B, V), torch.float32, h)
    _check(lib().amq_lm_sequence(_dev(Ep, torch.int32), _dev(alpha_e, torch.float32), vocab, E,
                                 _dev(Wxp, torch.int32), _dev(alpha_x, torch.float32), _dev(Whp, torch.int32),
                                 _dev(alpha_h, torch.float32), H, k_w, _opt(bias), _dev(Wsp, torch.int32),
                                 _dev(alpha_s, torch.float32), V, k_ws, _opt(bias_s), _dev(ids, torch.int64), steps,
                                 _dev(h, torch.float32), _dev(c, torch.float32), B, k_a, k_as, T,
                                 _dev(logprob, torch.float32), ws.data_ptr(), ws.numel(), _stream()))
    return logprob


def lm_sequence_score(Ep, alpha_e, E, Wxp, alpha_x, Whp, alpha_h, H, bias, Wsp, alpha_s, bias_s, ids, targets, h, c,
                      k_a, k_as, T, ws=None, out=None):
    """ids, targets [steps, B] -> log-probability of targets[t, b] at step t, [steps, B]; h, c updated in place."""
    vocab = Ep.shape[1]
    k_w = Wxp.shape[0]
    k_ws, V, _ = Wsp.shape
    steps, B = ids.shape
    if tuple(targets.shape) != (steps, B):
        raise AmqError("targets must have the shape of ids")
    if ws is None:
        ws = torch.empty(int(lib().amq_lm_sequence_score_workspace_bytes(E, H, V, B, k_a, k_as)), dtype=torch.uint8,
                         device=h.device)
    if out is None:
        out = _empty((steps, B), torch.float32, h)
    _check(lib().amq_lm_sequence_score(_dev(Ep, torch.int32), _dev(alpha_e, torch.float32), vocab, E,
                                       _dev(Wxp, torch.int32), _dev(alpha_x, torch.float32), _dev(Whp, torch.int32),
                                       _dev(alpha_h, torch.float32), H, k_w, _opt(bias), _dev(Wsp, torch.int32),
                                       _dev(alpha_s, torch.float32), V, k_ws, _opt(bias_s), _dev(ids, torch.int64),
                                       _dev(targets, torch.int64), steps, _dev(h, torch.float32),
                                       _dev(c, torch.float32), B, k_a, k_as, T, _dev(out, torch.float32),
                                       ws.data_ptr(), ws.numel(), _stream()))
    return out


def quantize_refined_greedy(W, k):
    """Refined greedy approximation of every row of W [rows, cols] -> planes [k, rows, wpr], alpha [rows, k]."""
    if W.dim() != 2 or W.stride(1) != 1 or W.dtype != torch.float32 or not W.is_cuda:
        raise AmqError("expected a 2-D float32 GPU tensor with unit column stride")
    rows, cols = W.shape
    planes = _empty((k, rows, wpr(cols)), torch.int32, W)
    alpha = _empty((rows, k), torch.float32, W)
    _check(lib().amq_quantize_refined_greedy(W.data_ptr(), rows, cols, W.stride(0), k, planes.data_ptr(),
                                             alpha.data_ptr(), _stream()))
    return planes, alpha


def quantize_ternary(W, T):
    """Ternary quantization of every row of W [rows, cols] as 2-bit codes with equal coefficients
    -> planes [2, rows, wpr], alpha [rows, 2]."""
    if W.dim() != 2 or W.stride(1) != 1 or W.dtype != torch.float32 or not W.is_cuda:
        raise AmqError("expected a 2-D float32 GPU tensor with unit column stride")
    rows, cols = W.shape
    planes = _empty((2, rows, wpr(cols)), torch.int32, W)
    alpha = _empty((rows, 2), torch.float32, W)
    _check(lib().amq_quantize_ternary(W.data_ptr(), rows, cols, W.stride(0), T, planes.data_ptr(),
                                      alpha.data_ptr(), _stream()))
    return planes, alpha


def relative_mse(W, planes, alpha):
    """Returns (result [3] = error, norm, error / norm; row_err [rows]; row_norm [rows]), float64 GPU tensors."""
    if W.dim() != 2 or W.stride(1) != 1 or W.dtype != torch.float32 or not W.is_cuda:
        raise AmqError("expected a 2-D float32 GPU tensor with unit column stride")
    rows, cols = W.shape
    k = planes.shape[0]
    row_err = _empty((rows,), torch.float64, W)
    row_norm = _empty((rows,), torch.float64, W)
    result = _empty((3,), torch.float64, W)
    _check(lib().amq_relative_mse(W.data_ptr(), rows, cols, W.stride(0), k, _dev(planes, torch.int32),
                                  _dev(alpha, torch.float32), row_err.data_ptr(), row_norm.data_ptr(),
                                  result.data_ptr(), _stream()))
    return result, row_err, row_norm


def dequantize(planes, alpha, cols, out=None):
    """Reconstruction [rows, cols] float32 of a row-wise quantization (planes [k, rows, wpr], alpha [rows, k])."""
    k, rows, _ = planes.shape
    if out is None:
        out = _empty((rows, cols), torch.float32, planes)
    if out.dim() != 2 or out.stride(1) != 1 or out.dtype != torch.float32 or not out.is_cuda:
        raise AmqError("expected a 2-D float32 GPU tensor with unit column stride")
    _check(lib().amq_dequantize(_dev(planes, torch.int32), _dev(alpha, torch.float32), rows, cols, k, out.data_ptr(),
                                out.stride(0), _stream()))
    return out


def clip_(w, lo=-1.0, hi=1.0):
    """Clips a contiguous float32 GPU tensor to [lo, hi] in place."""
    _check(lib().amq_clip(_dev(w, torch.float32), w.numel(), lo, hi, _stream()))
    return w


class _FakeQuantize(torch.autograd.Function):
    """w -> w_hat = sum_i alpha_i b_i (row-wise alternating quantization) with the straight-through
    gradient of Sec. 4: d f / d w = d f / d w_hat.  Both directions are argument marshalling: the
    forward pass is two library calls, the backward pass returns its argument."""

    @staticmethod
    def forward(ctx, W, k, T):
        planes, alpha = quantize_weights(W.detach().contiguous(), k, T)
        return dequantize(planes, alpha, W.shape[1])

    @staticmethod
    def backward(ctx, grad):
        return grad, None, None


def fake_quantize(W, k, T=2):
    return _FakeQuantize.apply(W, k, T)
