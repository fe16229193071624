"""numpy front end of the CPU oracle (oracle/amq_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The GPU package never imports this module, and
this module never imports the GPU package.  Every function is argument
marshalling around one C function of the same name; the arithmetic and its
citations live in the C file.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None

_f32p = np.ctypeslib.ndpointer(dtype=np.float32, flags="C_CONTIGUOUS")
_u8p = np.ctypeslib.ndpointer(dtype=np.uint8, flags="C_CONTIGUOUS")
_u32p = np.ctypeslib.ndpointer(dtype=np.uint32, flags="C_CONTIGUOUS")
_i32p = np.ctypeslib.ndpointer(dtype=np.int32, flags="C_CONTIGUOUS")
_f64p = np.ctypeslib.ndpointer(dtype=np.float64, flags="C_CONTIGUOUS")
_i64p = np.ctypeslib.ndpointer(dtype=np.int64, flags="C_CONTIGUOUS")
_i64 = C.c_int64
_int = C.c_int


def lib():
    global _lib
    if _lib is None:
        # AMQ_ORACLE_SANITIZE=1 (set by the sanitizer test for its child process) selects the build
        # under AddressSanitizer / UndefinedBehaviorSanitizer
        path = _build.build(sanitize=os.environ.get("AMQ_ORACLE_SANITIZE") == "1")
        L = C.CDLL(path)
        L.amq_oracle_set_threads.argtypes = [_int]
        L.amq_oracle_get_threads.restype = _int
        L.amq_oracle_wpr.argtypes = [_i64]
        L.amq_oracle_wpr.restype = _i64
        L.amq_oracle_greedy.argtypes = [_f32p, _i64, _int, _u8p, _f32p]
        L.amq_oracle_ls.argtypes = [_f32p, _i64, _int, _u8p, _f32p]
        L.amq_oracle_ls.restype = _int
        L.amq_oracle_code_table.argtypes = [_f32p, _int, _f32p, _i32p, _f32p]
        L.amq_oracle_bst.argtypes = [_f32p, _i64, _int, _f32p, _u8p]
        L.amq_oracle_error.argtypes = [_f32p, _i64, _int, _u8p, _f32p]
        L.amq_oracle_error.restype = C.c_double
        L.amq_oracle_quantize.argtypes = [_f32p, _i64, _int, _int, _u8p, _f32p, C.c_void_p]
        L.amq_oracle_pack.argtypes = [_u8p, _i64, _u32p]
        L.amq_oracle_quantize_rows.argtypes = [_f32p, _i64, _i64, _i64, _int, _int, _u32p, _f32p]
        L.amq_oracle_binary_dots.argtypes = [_u32p, _i64, _i64, _int, _u32p, _i64, _int, _i32p]
        L.amq_oracle_binary_gemm.argtypes = [_u32p, _f32p, _i64, _i64, _int, _u32p, _f32p, _i64, _int,
                                             C.c_void_p, _int, _f32p]
        L.amq_oracle_lstm_step.argtypes = [_u32p, _f32p, _u32p, _f32p, _i64, _i64, _int, C.c_void_p,
                                           _f32p, _f32p, _f32p, _i64, _int, _int, _f32p, _f32p]
        L.amq_oracle_gru_step.argtypes = [_u32p, _f32p, _u32p, _f32p, _i64, _i64, _int, C.c_void_p,
                                          C.c_void_p, _f32p, _f32p, _i64, _int, _int, _f32p]
        L.amq_oracle_embedding_lookup.argtypes = [_u32p, _f32p, _i64, _i64, _int, _i64p, _i64, _u32p, _f32p]
        L.amq_oracle_lstm_step_xq.argtypes = [_u32p, _f32p, _u32p, _f32p, _i64, _i64, _int, C.c_void_p,
                                              _u32p, _f32p, _f32p, _f32p, _i64, _int, _int, _f32p, _f32p]
        L.amq_oracle_log_softmax.argtypes = [_f32p, _i64, _i64, _f32p]
        L.amq_oracle_softmax_layer.argtypes = [_u32p, _f32p, _i64, _i64, _int, C.c_void_p, _f32p, _i64,
                                               _int, _int, _f32p, _f32p]
        L.amq_oracle_quantize_rows_final_ls.argtypes = [_f32p, _i64, _i64, _i64, _int, _int, _u32p, _f32p]
        L.amq_oracle_dequantize.argtypes = [_u32p, _f32p, _i64, _i64, _int, _f32p, _i64]
        L.amq_oracle_clip.argtypes = [_f32p, _i64, C.c_float, C.c_float]
        L.amq_oracle_refined_greedy.argtypes = [_f32p, _i64, _int, _u8p, _f32p]
        L.amq_oracle_refined_greedy_rows.argtypes = [_f32p, _i64, _i64, _i64, _int, _u32p, _f32p]
        L.amq_oracle_ternary.argtypes = [_f32p, _i64, _int, _u8p, _f32p]
        L.amq_oracle_ternary_rows.argtypes = [_f32p, _i64, _i64, _i64, _int, _u32p, _f32p]
        L.amq_oracle_relative_mse.argtypes = [_f32p, _i64, _i64, _i64, _int, _u32p, _f32p, _f64p, _f64p]
        L.amq_oracle_relative_mse.restype = C.c_double
        L.amq_oracle_gru_step_rb.argtypes = [_u32p, _f32p, _u32p, _f32p, _i64, _i64, _int, C.c_void_p,
                                             C.c_void_p, _f32p, _f32p, _i64, _int, _int, C.c_void_p, _f32p, _f32p]
        L.amq_oracle_gamma.argtypes = [C.c_double] * 4
        L.amq_oracle_gamma.restype = C.c_double
        _lib = L
    return _lib


def set_threads(t: int) -> int:
    lib().amq_oracle_set_threads(int(t))
    return lib().amq_oracle_get_threads()


def host_threads() -> int:
    """Threads the host offers this process (its CPU affinity)."""
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count() or 1


def wpr(n: int) -> int:
    return int(lib().amq_oracle_wpr(int(n)))


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _opt(a):
    if a is None:
        return None, None
    a = _f32(a)
    return a, a.ctypes.data_as(C.c_void_p)


def greedy(w, k):
    w = _f32(w)
    n = w.shape[0]
    code = np.zeros((k, n), np.uint8)
    alpha = np.zeros(k, np.float32)
    lib().amq_oracle_greedy(w, n, k, code, alpha)
    return code, alpha


def ls(w, code, alpha):
    """Returns (alpha_new, solved)."""
    w = _f32(w)
    code = np.ascontiguousarray(code, np.uint8)
    k, n = code.shape
    alpha = _f32(alpha).copy()
    ok = lib().amq_oracle_ls(w, n, k, code, alpha)
    return alpha, bool(ok)


def code_table(alpha):
    alpha = _f32(alpha)
    k = alpha.shape[0]
    v = np.zeros(1 << k, np.float32)
    pat = np.zeros(1 << k, np.int32)
    mid = np.zeros(1 << k, np.float32)
    lib().amq_oracle_code_table(alpha, k, v, pat, mid)
    return v, pat, mid[: (1 << k) - 1]


def bst(w, alpha):
    w = _f32(w)
    alpha = _f32(alpha)
    k, n = alpha.shape[0], w.shape[0]
    code = np.zeros((k, n), np.uint8)
    lib().amq_oracle_bst(w, n, k, alpha, code)
    return code


def error(w, code, alpha):
    w = _f32(w)
    code = np.ascontiguousarray(code, np.uint8)
    k, n = code.shape
    return float(lib().amq_oracle_error(w, n, k, code, _f32(alpha)))


def quantize(w, k, T, trace=False):
    w = _f32(w)
    n = w.shape[0]
    code = np.zeros((k, n), np.uint8)
    alpha = np.zeros(k, np.float32)
    tr = np.zeros(1 + 2 * T, np.float64) if trace else None
    lib().amq_oracle_quantize(w, n, k, T, code, alpha, tr.ctypes.data_as(C.c_void_p) if trace else None)
    return (code, alpha, tr) if trace else (code, alpha)


def pack(code_plane):
    code_plane = np.ascontiguousarray(code_plane, np.uint8)
    n = code_plane.shape[0]
    words = np.zeros(wpr(n), np.uint32)
    lib().amq_oracle_pack(code_plane, n, words)
    return words


def quantize_rows(W, k, T):
    """W [rows, cols] -> planes [k, rows, wpr] uint32, alpha [rows, k] float32."""
    W = _f32(W)
    rows, cols = W.shape
    planes = np.zeros((k, rows, wpr(cols)), np.uint32)
    alpha = np.zeros((rows, k), np.float32)
    lib().amq_oracle_quantize_rows(W, rows, cols, cols, k, T, planes, alpha)
    return planes, alpha


def binary_dots(Wp, n, Xp):
    """Wp [k_w, m, wpr], Xp [k_a, batch, wpr] -> D [batch, m, k_w, k_a] int32."""
    Wp = np.ascontiguousarray(Wp, np.uint32)
    Xp = np.ascontiguousarray(Xp, np.uint32)
    k_w, m, _ = Wp.shape
    k_a, batch, _ = Xp.shape
    D = np.zeros((batch, m, k_w, k_a), np.int32)
    lib().amq_oracle_binary_dots(Wp, m, n, k_w, Xp, batch, k_a, D)
    return D


def binary_gemm(Wp, alpha, n, Xp, beta, bias=None, Y=None):
    """Y [batch, m].  If Y is given the product is added to it (accumulate)."""
    Wp = np.ascontiguousarray(Wp, np.uint32)
    Xp = np.ascontiguousarray(Xp, np.uint32)
    k_w, m, _ = Wp.shape
    k_a, batch, _ = Xp.shape
    acc = Y is not None
    out = _f32(Y).copy() if acc else np.zeros((batch, m), np.float32)
    bias_a, bias_p = _opt(bias)
    lib().amq_oracle_binary_gemm(Wp, _f32(alpha), m, n, k_w, Xp, _f32(beta), batch, k_a, bias_p,
                                 1 if acc else 0, out)
    return out


def lstm_step(Wxp, alpha_x, Whp, alpha_h, I, H, bias, x, h_prev, c_prev, k_a, T):
    Wxp = np.ascontiguousarray(Wxp, np.uint32)
    Whp = np.ascontiguousarray(Whp, np.uint32)
    k_w = Wxp.shape[0]
    x, h_prev, c_prev = _f32(x), _f32(h_prev), _f32(c_prev)
    B = x.shape[0]
    h = np.zeros((B, H), np.float32)
    c = np.zeros((B, H), np.float32)
    bias_a, bias_p = _opt(bias)
    lib().amq_oracle_lstm_step(Wxp, _f32(alpha_x), Whp, _f32(alpha_h), I, H, k_w, bias_p, x, h_prev,
                               c_prev, B, k_a, T, h, c)
    return h, c


def gru_step(Wxp, alpha_x, Whp, alpha_h, I, H, bias_x, bias_h, x, h_prev, k_a, T):
    Wxp = np.ascontiguousarray(Wxp, np.uint32)
    Whp = np.ascontiguousarray(Whp, np.uint32)
    k_w = Wxp.shape[0]
    x, h_prev = _f32(x), _f32(h_prev)
    B = x.shape[0]
    h = np.zeros((B, H), np.float32)
    bx_a, bx_p = _opt(bias_x)
    bh_a, bh_p = _opt(bias_h)
    lib().amq_oracle_gru_step(Wxp, _f32(alpha_x), Whp, _f32(alpha_h), I, H, k_w, bx_p, bh_p, x, h_prev,
                              B, k_a, T, h)
    return h


def embedding_lookup(Ep, alpha_e, n, ids):
    """Ep [k, vocab, wpr], alpha_e [vocab, k], ids [B] -> Xp [k, B, wpr], beta [B, k]."""
    Ep = np.ascontiguousarray(Ep, np.uint32)
    ids = np.ascontiguousarray(ids, np.int64)
    k, vocab, w = Ep.shape
    B = ids.shape[0]
    if ids.min() < 0 or ids.max() >= vocab:
        raise ValueError("id out of range")
    Xp = np.zeros((k, B, w), np.uint32)
    beta = np.zeros((B, k), np.float32)
    lib().amq_oracle_embedding_lookup(Ep, _f32(alpha_e), vocab, n, k, ids, B, Xp, beta)
    return Xp, beta


def lstm_step_xq(Wxp, alpha_x, Whp, alpha_h, I, H, bias, Xp, beta_x, h_prev, c_prev, T):
    """LSTM step with x_t given as packed planes Xp [k_a, B, wpr(I)] + beta_x [B, k_a]."""
    Wxp = np.ascontiguousarray(Wxp, np.uint32)
    Whp = np.ascontiguousarray(Whp, np.uint32)
    Xp = np.ascontiguousarray(Xp, np.uint32)
    k_w = Wxp.shape[0]
    k_a, B, _ = Xp.shape
    h_prev, c_prev = _f32(h_prev), _f32(c_prev)
    h = np.zeros((B, H), np.float32)
    c = np.zeros((B, H), np.float32)
    bias_a, bias_p = _opt(bias)
    lib().amq_oracle_lstm_step_xq(Wxp, _f32(alpha_x), Whp, _f32(alpha_h), I, H, k_w, bias_p, Xp,
                                  _f32(beta_x), h_prev, c_prev, B, k_a, T, h, c)
    return h, c


def log_softmax(Y):
    Y = _f32(Y)
    B, V = Y.shape
    out = np.zeros((B, V), np.float32)
    lib().amq_oracle_log_softmax(Y, B, V, out)
    return out


def softmax_layer(Wsp, alpha_s, H, bias, h, k_a, T):
    """Returns (logits, logprob), each [B, V] float32."""
    Wsp = np.ascontiguousarray(Wsp, np.uint32)
    k_w, V, _ = Wsp.shape
    h = _f32(h)
    B = h.shape[0]
    logits = np.zeros((B, V), np.float32)
    logprob = np.zeros((B, V), np.float32)
    bias_a, bias_p = _opt(bias)
    lib().amq_oracle_softmax_layer(Wsp, _f32(alpha_s), V, H, k_w, bias_p, h, B, k_a, T, logits, logprob)
    return logits, logprob


def quantize_rows_final_ls(W, k, T):
    """Alg. 2 followed by one more coefficient update (Eq. 5) on the final codes."""
    W = _f32(W)
    rows, cols = W.shape
    planes = np.zeros((k, rows, wpr(cols)), np.uint32)
    alpha = np.zeros((rows, k), np.float32)
    lib().amq_oracle_quantize_rows_final_ls(W, rows, cols, cols, k, T, planes, alpha)
    return planes, alpha


def dequantize(planes, alpha, cols):
    """Reconstruction [rows, cols] float32 of a row-wise quantization."""
    planes = np.ascontiguousarray(planes, np.uint32)
    k, rows, _ = planes.shape
    out = np.zeros((rows, cols), np.float32)
    lib().amq_oracle_dequantize(planes, _f32(alpha), rows, cols, k, out, cols)
    return out


def clip(w, lo=-1.0, hi=1.0):
    out = _f32(w).copy()
    lib().amq_oracle_clip(out.reshape(-1), out.size, lo, hi)
    return out


def refined_greedy(w, k):
    """Refined greedy approximation of one vector: code [k, n] uint8 (1 = +1), alpha [k]."""
    w = _f32(w)
    n = w.shape[0]
    code = np.zeros((k, n), np.uint8)
    alpha = np.zeros(k, np.float32)
    lib().amq_oracle_refined_greedy(w, n, k, code, alpha)
    return code, alpha


def refined_greedy_rows(W, k):
    W = _f32(W)
    rows, cols = W.shape
    planes = np.zeros((k, rows, wpr(cols)), np.uint32)
    alpha = np.zeros((rows, k), np.float32)
    lib().amq_oracle_refined_greedy_rows(W, rows, cols, cols, k, planes, alpha)
    return planes, alpha


def ternary(w, T):
    """Ternary quantization of one vector as constrained 2-bit codes: code [2, n] uint8 (1 = +1), alpha [2]
    with alpha[0] == alpha[1]; the ternary value of an entry is (alpha[0] + alpha[1]) * t."""
    w = _f32(w)
    n = w.shape[0]
    code = np.zeros((2, n), np.uint8)
    alpha = np.zeros(2, np.float32)
    lib().amq_oracle_ternary(w, n, T, code, alpha)
    return code, alpha


def ternary_rows(W, T):
    W = _f32(W)
    rows, cols = W.shape
    planes = np.zeros((2, rows, wpr(cols)), np.uint32)
    alpha = np.zeros((rows, 2), np.float32)
    lib().amq_oracle_ternary_rows(W, rows, cols, cols, T, planes, alpha)
    return planes, alpha


def relative_mse(W, planes, alpha):
    """(ratio, row_err [rows], row_norm [rows]) of a row-wise quantization, binary64."""
    W = _f32(W)
    rows, cols = W.shape
    planes = np.ascontiguousarray(planes, np.uint32)
    k = planes.shape[0]
    row_err = np.zeros(rows, np.float64)
    row_norm = np.zeros(rows, np.float64)
    ratio = lib().amq_oracle_relative_mse(W, rows, cols, cols, k, planes, _f32(alpha), row_err, row_norm)
    return float(ratio), row_err, row_norm


def gru_step_reset_before(Wxp, alpha_x, Whp, alpha_h, I, H, bias_x, bias_h, x, h_prev, k_a, T, g=None,
                          return_g=False):
    """g (optional): use this r * h_prev instead of computing it.  return_g: also return the one used."""
    Wxp = np.ascontiguousarray(Wxp, np.uint32)
    Whp = np.ascontiguousarray(Whp, np.uint32)
    k_w = Wxp.shape[0]
    x, h_prev = _f32(x), _f32(h_prev)
    B = x.shape[0]
    h = np.zeros((B, H), np.float32)
    bx_a, bx_p = _opt(bias_x)
    bh_a, bh_p = _opt(bias_h)
    g_a, g_p = _opt(g)
    g_used = np.zeros((B, H), np.float32)
    lib().amq_oracle_gru_step_rb(Wxp, _f32(alpha_x), Whp, _f32(alpha_h), I, H, k_w, bx_p, bh_p, x, h_prev,
                                 B, k_a, T, g_p, g_used, h)
    return (h, g_used) if return_g else h


def gamma(m, n, k_w, k_h):
    return float(lib().amq_oracle_gamma(m, n, k_w, k_h))
