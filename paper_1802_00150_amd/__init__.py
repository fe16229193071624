"""MI355X (gfx950) library for alternating multi-bit quantization and the quantized LSTM / GRU
inference step (arXiv 1802.00150).

`binding` wraps the C ABI of include/amq.h (libamq.so, built from csrc/ by `build`);
`inputs` holds the seeded synthetic workloads.  Importing the package loads nothing; the
shared library is loaded at the first call and a missing library is an error, never a fallback.
"""
from . import binding  # noqa: F401
from .binding import (AmqError, clip_, dequantize, fake_quantize, binary_dots, binary_gemm, binary_gemv, binary_gemv_grouped, bst_assign,  # noqa: F401
                      embedding_lookup, gru_sequence, gru_sequence_workspace, gru_step, gru_step_reset_before, gru_workspace, lm_sequence, lm_sequence_score, lm_step, lm_workspace, log_softmax, ls_update,
                      lstm_sequence, lstm_sequence_abandoned, lstm_sequence_workspace, lstm_step, lstm_step_packed, lstm_step_packed_grouped, lstm_step_static, stream_read_probe, lstm_workspace, quantize_activations,
                      quantize_refined_greedy, quantize_ternary, quantize_weights, relative_mse, softmax_layer, softmax_layer_workspace, version, wpr)
