/*
 * amq.h -- C ABI of the MI355X (gfx950) library for alternating multi-bit
 * quantization and the quantized LSTM / GRU inference step built on it
 * (arXiv 1802.00150).
 *
 * Conventions (all entry points):
 *   - Every pointer is a DEVICE pointer unless its comment says "host".
 *   - The caller owns every buffer, including workspaces.  The library
 *     allocates nothing and keeps no results between calls (it remembers, per
 *     device, which kernels it has configured and where its static scratch
 *     lies).  Inputs are never modified.  Outputs must not alias inputs unless
 *     stated.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work; they never synchronise the host.
 *   - Return value: AMQ_OK, or an error code.  Arguments are validated on the
 *     host before anything is launched, so AMQ_ERR_INVALID / AMQ_ERR_UNSUPPORTED
 *     leave the device untouched.  No C++ exception crosses this boundary.
 *   - Inputs must be finite; NaN / Inf give unspecified results.
 *
 * Packed code layout (the exchange format for every `planes` argument):
 *   a k-bit quantization of `rows` vectors of length n is k bit-planes of
 *   uint32 words, indexed [plane][row][word], with wpr = amq_wpr(n) =
 *   4 * ceil(n / 128) words per row (rows are 16-byte aligned).  Entry l of a
 *   row is bit (l % 32) of word (l / 32); bit 1 means +1, bit 0 means -1.
 *   Bits at positions >= n are 0 in every operand.  Plane i (0-based) pairs
 *   with coefficient i of that row: coef[row * k + i].
 */
#ifndef AMQ_H_
#define AMQ_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AMQ_OK 0
#define AMQ_ERR_INVALID 1     /* null pointer, k outside 1..4, T < 0, non-positive size, bad workspace */
#define AMQ_ERR_UNSUPPORTED 2 /* a size beyond the limits below */
#define AMQ_ERR_HIP 3         /* HIP runtime error; see amq_last_hip_error() */

#define AMQ_MAX_BITS 4
#define AMQ_MAX_QUANT_N 16384 /* longest vector the quantizers accept */
#define AMQ_MAX_DOT_N (1 << 20) /* longest vector the binary products accept */

/* Host-only helpers. */
int64_t amq_wpr(int64_t n);               /* words per row per plane, 4 * ceil(n / 128) */
const char* amq_version(void);
const char* amq_status_string(int status);
int amq_last_hip_error(void);             /* hipError_t of the last AMQ_ERR_HIP on this thread */

/*
 * Row-wise alternating multi-bit quantization of a weight matrix (Sec. 4: every
 * row gets its own coefficients; Alg. 2 on every row): greedy initialisation (Eq. 4), then T
 * times { least-squares coefficients (Eq. 5); sorted code table; binary-search
 * code assignment (Alg. 1) }.  No trailing least-squares step.  T = 0 returns
 * the greedy result.  If the k x k Gram matrix of the codes is singular the
 * coefficient update of that cycle is skipped.
 *   W      [rows][ld] float, ld >= cols (row stride in elements)
 *   planes [k][rows][wpr(cols)] uint32 out
 *   alpha  [rows][k] float out
 * Throughput-oriented: one wavefront (or one workgroup) per row.
 */
int amq_quantize_weights(const float* W, int64_t rows, int64_t cols, int64_t ld, int k, int T,
                         uint32_t* planes, float* alpha, void* stream);

/*
 * On-line quantization of a batch of activation vectors (Sec. 4: h_t depends on
 * the input and has to be quantized at inference time); the same mathematics as amq_quantize_weights on the
 * rows of X, X dense [batch][n].
 *   planes [k][batch][wpr(n)] uint32 out,  beta [batch][k] float out
 */
int amq_quantize_activations(const float* X, int64_t batch, int64_t n, int k, int T,
                             uint32_t* planes, float* beta, void* stream);

/*
 * Staged hooks of the quantizer (for step-by-step parity checks):
 *   amq_ls_update : Eq. 5 with the codes given; coef [rows][k] is updated in
 *                   place (left unchanged for a row whose Gram matrix is singular).
 *   amq_bst_assign: Alg. 1 for every entry with the coefficients given.
 */
int amq_ls_update(const float* X, int64_t rows, int64_t n, int k, const uint32_t* planes,
                  float* coef, void* stream);
int amq_bst_assign(const float* X, int64_t rows, int64_t n, int k, const float* coef,
                   uint32_t* planes, void* stream);

/*
 * Binary inner products (App. A: XNOR then bit count) of every weight plane
 * with every activation plane:
 *   D[b][r][i][j] = sum_l Bw_i[r][l] * c_j[b][l] = n - 2 * popcount(Bw_i[r] xor c_j[b])
 *   Wp [k_w][m][wpr(n)],  Xp [k_a][batch][wpr(n)],  D [batch][m][k_w][k_a] int32 out
 */
int amq_binary_dots(const uint32_t* Wp, int64_t m, int64_t n, int k_w, const uint32_t* Xp,
                    int64_t batch, int k_a, int32_t* D, void* stream);

/*
 * Quantized matrix product (Sec. 4, Fig. 3): binary products first, then the
 * coefficients,
 *   Y[b][r] = (accumulate ? Y[b][r] : 0) + bias[r]
 *             + sum_i alpha[r][i] * sum_j beta[b][j] * D[b][r][i][j].
 *   alpha [m][k_w], beta [batch][k_a], bias [m] or NULL, Y [batch][m] float.
 * amq_binary_gemv is the batch-1 case (memory-bound streaming of the weight
 * planes); amq_binary_gemm takes any batch.
 */
int amq_binary_gemv(const uint32_t* Wp, const float* alpha, int64_t m, int64_t n, int k_w,
                    const uint32_t* Xp, const float* beta, int k_a, const float* bias,
                    int accumulate, float* Y, void* stream);
int amq_binary_gemm(const uint32_t* Wp, const float* alpha, int64_t m, int64_t n, int k_w,
                    const uint32_t* Xp, const float* beta, int64_t batch, int k_a,
                    const float* bias, int accumulate, float* Y, void* stream);

/*
 * `groups` independent batch-1 products in one launch, group g using
 *   Wp + g * k_w * m * wpr, alpha + g * m * k_w, Xp + g * k_a * wpr,
 *   beta + g * k_a, Y + g * m   (bias, if given, is shared).
 * This is how the memory-bound product is measured from HBM rather than from
 * cache: many matrices of the benchmark's shape, each read once.
 */
int amq_binary_gemv_grouped(int64_t groups, const uint32_t* Wp, const float* alpha, int64_t m,
                            int64_t n, int k_w, const uint32_t* Xp, const float* beta, int k_a,
                            const float* bias, float* Y, void* stream);

/*
 * One quantized LSTM step (Eq. 6).  Wx is 4H x I and Wh is 4H x H, each
 * row-wise k_w-bit (planes + alpha as produced by amq_quantize_weights); gate
 * row blocks in the order i, f, o, g; sigmoid for i, f, o and tanh for g.
 * x_t and h_{t-1} are quantized on line to k_a bits with T alternating cycles,
 * each vector on its own.
 *   bias [4H] (b_i + b_h) or NULL;  x [B][I];  h_prev, c_prev, h_out, c_out [B][H]
 *   h_out may alias h_prev and c_out may alias c_prev.
 *   workspace: at least amq_lstm_workspace_bytes(I, H, B, k_a) bytes, 256-byte aligned.
 */
size_t amq_lstm_workspace_bytes(int64_t I, int64_t H, int64_t B, int k_a);
int amq_lstm_step(const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp,
                  const float* alpha_h, int64_t I, int64_t H, int k_w, const float* bias,
                  const float* x, const float* h_prev, const float* c_prev, int64_t B, int k_a,
                  int T, float* h_out, float* c_out, void* workspace, size_t workspace_bytes,
                  void* stream);

/*
 * amq_lstm_step for callers that cannot allocate or hand over a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments without the
 * workspace, same arithmetic and results.  The scratch memory is a static device array of
 * AMQ_STATIC_SCRATCH_BYTES inside the library (every GPU the library runs on holds its own copy
 * until the process ends); the call itself allocates nothing.  Shapes whose
 * amq_lstm_workspace_bytes(I, H, B, k_a) exceeds AMQ_STATIC_SCRATCH_BYTES return
 * AMQ_ERR_UNSUPPORTED.  All calls on one GPU share that GPU's array: calls that may overlap in
 * time on one GPU (different streams, different host threads) race and must be serialised by
 * the caller.  Nothing in the array is carried from one call to the next.
 */
#define AMQ_STATIC_SCRATCH_BYTES (4u << 20)
int amq_lstm_step_static(const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp,
                         const float* alpha_h, int64_t I, int64_t H, int k_w, const float* bias,
                         const float* x, const float* h_prev, const float* c_prev, int64_t B, int k_a,
                         int T, float* h_out, float* c_out, void* stream);

/*
 * The same LSTM step on operands that are already quantized: x_t as packed planes Xp
 * [k_a][B][wpr(I)] with beta_x [B][k_a] (Sec. 4: with one-hot inputs x_t is a row of the
 * quantized embedding matrix, so it arrives already quantized), h_{t-1} as Hp / beta_h.
 * Products, coefficient epilogue and cell only; no workspace.  Returns AMQ_ERR_UNSUPPORTED for
 * I or H above AMQ_MAX_QUANT_N.
 */
int amq_lstm_step_packed(const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp,
                         const float* alpha_h, int64_t I, int64_t H, int k_w, const float* bias,
                         const uint32_t* Xp, const float* beta_x, const uint32_t* Hp,
                         const float* beta_h, const float* c_prev, int64_t B, int k_a, float* h_out,
                         float* c_out, void* stream);

/*
 * `groups` independent batch-1 LSTM steps on quantized operands in one launch (the recurrent
 * counterpart of amq_binary_gemv_grouped: how the memory-bound batch-1 step -- the case App. A times --
 * is measured with every weight plane coming from HBM rather than from cache).  Group g uses
 *   Wxp + g * k_w * 4H * wpr(I), alpha_x + g * 4H * k_w, Whp + g * k_w * 4H * wpr(H), alpha_h + g * 4H * k_w,
 *   Xp + g * k_a * wpr(I), beta_x + g * k_a, Hp + g * k_a * wpr(H), beta_h + g * k_a,
 *   c_prev, h_out, c_out + g * H;  bias [4H] (nullable) is shared.
 * Same arithmetic as amq_lstm_step_packed with B = 1 on every group.  groups <= 65535; I, H <= 8192.
 */
int amq_lstm_step_packed_grouped(int64_t groups, const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp,
                                 const float* alpha_h, int64_t I, int64_t H, int k_w, const float* bias,
                                 const uint32_t* Xp, const float* beta_x, const uint32_t* Hp,
                                 const float* beta_h, const float* c_prev, int k_a, float* h_out,
                                 float* c_out, void* stream);

/*
 * Bandwidth yardstick (not part of the method): reads buf[0 .. bytes) once with 16-byte loads and
 * leaves an xor checksum per workgroup in sink (device, AMQ_STREAM_PROBE_SINK_WORDS 64-bit words).
 * bytes must be a multiple of 16, buf 16-byte aligned.  Timed over a buffer larger than the last-level
 * cache it gives the read rate this GPU sustains, the practical ceiling next to the nominal HBM peak.
 */
#define AMQ_STREAM_PROBE_SINK_WORDS 4096
int amq_stream_read_probe(const void* buf, size_t bytes, void* sink, void* stream);

/*
 * `steps` consecutive LSTM steps in one call (the recurrence of Eq. 6 over a
 * sequence): xs [steps][B][I]; h and c [B][H] are read as the initial state and
 * overwritten with the final state; hs [steps][B][H] (nullable) receives every
 * h_t.  Same arithmetic as `steps` calls of amq_lstm_step.
 * For B = 1 with I, H <= 1024 and 2- or 3-bit codes the recurrence runs inside one
 * launch that occupies the whole chip (pieces of 64 steps), the workgroups exchanging
 * h_t through the workspace.  That launch needs all its workgroups resident at once:
 * do not run it concurrently with other work that keeps compute units busy.  Its waits
 * are bounded.  If one gives up, the return value is still AMQ_OK (the launches were
 * issued; the outcome is only known on the device): h and c hold the state after the
 * last 64-step piece that completed (the initial state if none did), the rows of hs
 * from the piece that gave up onwards hold NaN, and the 32-bit word
 * at byte amq_lstm_sequence_flag_offset(...) of the workspace is non-zero.  A caller
 * that needs to know reads that word after synchronising the stream (it is zero after a
 * completed call; SIZE_MAX: this shape has no such word).
 */
size_t amq_lstm_sequence_flag_offset(int64_t I, int64_t H, int64_t B, int k_a);
/*
 * Workspace with which amq_lstm_sequence takes W_x x_t off the recurrent chain for B > 1 (Eq. 6: the
 * inputs do not depend on the recurrence): amq_lstm_workspace_bytes plus room for the codes of two
 * consecutive inputs and the x-side sums of one step.  With a smaller workspace (at least
 * amq_lstm_workspace_bytes) the call runs the steps one after the other; the results are the same bit
 * for bit.
 */
size_t amq_lstm_sequence_workspace_bytes(int64_t I, int64_t H, int64_t B, int k_a);
int amq_lstm_sequence(const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp,
                      const float* alpha_h, int64_t I, int64_t H, int k_w, const float* bias,
                      const float* xs, int64_t steps, float* h, float* c, int64_t B, int k_a, int T,
                      float* hs, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Test hook for the give-up path above: the number of polls after which a wait of the
 * one-launch recurrence gives up, for launches issued from now on (process-wide; 0
 * restores the default of 2^19).  With 1 the first wait that is not satisfied at once
 * gives up, every workgroup leaves, and the documented failure state results without
 * any kernel hanging.
 */
void amq_debug_set_sequence_spin_limit(unsigned polls);

/*
 * Measurement hook: one of the two launches of a steady-state step of the batched amq_lstm_sequence
 * path, on its own, so that each can be timed and profiled under its own name.  half = 0: the front
 * launch (quantizes h and x_next, forms the x-side sums from the input codes the workspace holds);
 * half = 1: the back launch (h-side sums + the stored x-side sums + cell; h and c updated in place).
 * workspace: one that an amq_lstm_sequence call of the same shape has used (at least
 * amq_lstm_sequence_workspace_bytes), so that the codes and sums it reads are valid numbers.  The results
 * are not a step of any sequence.  AMQ_ERR_UNSUPPORTED where the sequence call would not take this path.
 */
int amq_debug_lstm_split_half(const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp,
                              const float* alpha_h, int64_t I, int64_t H, int k_w, const float* bias,
                              const float* x_next, float* h, float* c, int64_t B, int k_a, int T,
                              void* workspace, size_t workspace_bytes, int half, void* stream);

/*
 * One quantized GRU step.  The paper evaluates GRUs (Tables 2-5) without
 * printing the cell; this is the textbook cell in the form where the reset
 * gate multiplies the hidden-side product of the candidate, so that one
 * quantization of h_{t-1} serves all gates:
 *   ax = Wx x + bias_x, ah = Wh h_prev + bias_h   (3H rows, blocks r, z, n)
 *   r = sigmoid(ax_r + ah_r), z = sigmoid(ax_z + ah_z), n = tanh(ax_n + r * ah_n),
 *   h = (1 - z) * n + z * h_prev.
 *   bias_x, bias_h [3H] or NULL; h_out may alias h_prev.
 */
size_t amq_gru_workspace_bytes(int64_t I, int64_t H, int64_t B, int k_a);
int amq_gru_step(const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp,
                 const float* alpha_h, int64_t I, int64_t H, int k_w, const float* bias_x,
                 const float* bias_h, const float* x, const float* h_prev, int64_t B, int k_a, int T,
                 float* h_out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * `steps` consecutive GRU steps (the cell of amq_gru_step) on inputs xs [steps][B][I] that are all given:
 * h [B][H] is read as the initial state and overwritten with the final one; hs (nullable)
 * [steps][B][H] receives every h_t.  Same arithmetic as `steps` calls of amq_gru_step, bit for bit.  Where
 * the shape allows (2 to 128 batch tiles of 16 on at most 2048 row-block x tile tasks, I, H <= 1024, codes
 * of at most 3 bits) and the workspace has amq_gru_sequence_workspace_bytes, the input products leave the
 * recurrent chain as in amq_lstm_sequence; otherwise, and with a workspace of only amq_gru_workspace_bytes,
 * the steps are launched one by one.
 *   workspace: at least amq_gru_workspace_bytes(I, H, B, k_a) bytes, 256-byte aligned.
 */
size_t amq_gru_sequence_workspace_bytes(int64_t I, int64_t H, int64_t B, int k_a);
int amq_gru_sequence(const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp,
                     const float* alpha_h, int64_t I, int64_t H, int k_w, const float* bias_x,
                     const float* bias_h, const float* xs, int64_t steps, float* h, int64_t B, int k_a,
                     int T, float* hs, void* workspace, size_t workspace_bytes, void* stream);

/*
 * GRU step in the original form of the cell (the reset gate multiplies the previous state
 * before the candidate's hidden-side product):
 *   r = sigmoid(ax_r + ah_r), z = sigmoid(ax_z + ah_z),
 *   n = tanh(ax_n + Wh_n q(r * h_prev) + bias_h_n),  h = (1 - z) * n + z * h_prev,
 * ax = Wx q(x) + bias_x, ah = Wh q(h_prev) + bias_h, q = on-line quantization (k_a bits, T cycles).
 * r * h_prev is quantized on line like any activation: a second quantization and a second,
 * dependent product per step (which amq_gru_step avoids).  Arguments as amq_gru_step; h_out must not
 * alias h_prev; g_out [B][H] (nullable) receives r * h_prev (for step-by-step parity checks);
 * workspace at least amq_gru_reset_before_workspace_bytes(I, H, B, k_a) bytes.
 */
size_t amq_gru_reset_before_workspace_bytes(int64_t I, int64_t H, int64_t B, int k_a);
int amq_gru_step_reset_before(const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp,
                              const float* alpha_h, int64_t I, int64_t H, int k_w, const float* bias_x,
                              const float* bias_h, const float* x, const float* h_prev, int64_t B,
                              int k_a, int T, float* h_out, float* g_out, void* workspace,
                              size_t workspace_bytes, void* stream);

/*
 * amq_quantize_weights with options.  AMQ_QUANT_FINAL_LS adds one more coefficient update
 * (Eq. 5) after the last code assignment, so that the coefficients returned are the
 * least-squares optimum for the codes returned (Alg. 2 as printed ends with the codes).
 * Unknown flag bits are AMQ_ERR_INVALID.
 */
#define AMQ_QUANT_FINAL_LS 1
int amq_quantize_weights_ex(const float* W, int64_t rows, int64_t cols, int64_t ld, int k, int T,
                            int flags, uint32_t* planes, float* alpha, void* stream);

/*
 * Training-side helpers (Sec. 4, "Training": the forward pass uses the quantized weights
 * w_hat = sum_i alpha_i b_i, the gradient with respect to w is taken equal to the gradient
 * with respect to w_hat, and the full-precision weights are clipped to [-1, 1]).
 *   amq_dequantize: out [rows][ld_out] (ld_out >= cols) receives w_hat of a row-wise
 *     quantization; an entry is the binary32 left-to-right sum of +-alpha[r][i].
 *   amq_clip: w[0..n) clipped to [lo, hi] in place.
 */
int amq_dequantize(const uint32_t* planes, const float* alpha, int64_t rows, int64_t cols, int k,
                   float* out, int64_t ld_out, void* stream);
int amq_clip(float* w, int64_t n, float lo, float hi, void* stream);

/*
 * Refined greedy approximation (Sec. 2; the strongest earlier method in Tables 1-2), every row
 * on its own: for j = 1..k plane j is the sign of the current residual and alpha_j its mean
 * absolute value (Eq. 4), then alpha_1..alpha_j are replaced by the least-squares solution for
 * the first j planes (Eq. 5) and the residual is rebuilt from them.  Codes are never revisited.
 * Arguments as amq_quantize_weights.  (The plain greedy approximation is amq_quantize_weights
 * with T = 0.)
 */
int amq_quantize_refined_greedy(const float* W, int64_t rows, int64_t cols, int64_t ld, int k,
                                uint32_t* planes, float* alpha, void* stream);

/*
 * Ternary quantization written as the 2-bit case with alpha_1 = alpha_2 (Sec. 2), every row on its
 * own: w ~ a t with t in {-1, 0, +1}.  Initial codes by the threshold rule cited there (entries
 * with |w| <= (0.7 / cols) ||w||_1 become 0, the others their sign), then T alternating cycles
 * { a = least-squares coefficient of the codes = mean of |w| over the non-zero entries;
 *   t = nearest of {-a, 0, +a}, i.e. sign(w) where |w| > a / 2 }; T = 0 returns the threshold rule
 * with its own least-squares coefficient.
 *   planes [2][rows][wpr] (device, out): t as two code planes (+1 -> 1,1; -1 -> 0,0; 0 -> 1,0),
 *   alpha [rows][2] (device, out): {a / 2, a / 2} -- the format of amq_quantize_weights with k = 2,
 *   so every product entry point takes the result as it is.  Other arguments and errors as
 *   amq_quantize_weights.
 */
int amq_quantize_ternary(const float* W, int64_t rows, int64_t cols, int64_t ld, int T, uint32_t* planes,
                         float* alpha, void* stream);

/*
 * Relative mean squared error of a row-wise quantization (the measure of Tables 1-2):
 *   result[0] = sum over the matrix of (W - sum_i alpha_i B_i)^2,  result[1] = sum of W^2,
 *   result[2] = result[0] / result[1];  row_err [rows], row_norm [rows] receive the two sums of
 *   every row.  All three outputs are device arrays of double.
 */
int amq_relative_mse(const float* W, int64_t rows, int64_t cols, int64_t ld, int k,
                     const uint32_t* planes, const float* alpha, double* row_err, double* row_norm,
                     double* result, void* stream);

/*
 * Embedding lookup (Eq. 6, first line; Sec. 4): with one-hot inputs W_e x_t is a row of the
 * embedding matrix, and a table quantized off line by amq_quantize_weights (Ep [k][vocab][wpr(n)],
 * alpha_e [vocab][k]) holds that row as a finished k-bit quantization.  Copies rows ids[0..B)
 * into operand form:
 *   ids [B] int64 (device);  Xp [k][B][wpr(n)] out;  beta [B][k] out.
 * An id outside [0, vocab) gives the zero vector (plane bits 0, coefficients 0); it is never
 * dereferenced.
 */
int amq_embedding_lookup(const uint32_t* Ep, const float* alpha_e, int64_t vocab, int64_t n, int k,
                         const int64_t* ids, int64_t B, uint32_t* Xp, float* beta, void* stream);

/*
 * Logarithm of the softmax of Eq. 6 (last line), for every row of Y [B][V]:
 *   out[b][v] = Y[b][v] - log(sum_u exp(Y[b][u])).
 * out may be Y itself.
 */
int amq_log_softmax(const float* Y, int64_t B, int64_t V, float* out, void* stream);

/*
 * Output layer of Eq. 6: log softmax(W_s h_t + b_s), W_s (V x H) row-wise k_w-bit, h_t quantized
 * on line to k_a bits (T cycles).  logprob [B][V] receives the logits first and is then normalised
 * in place.  workspace: at least amq_softmax_layer_workspace_bytes(V, H, B, k_a) bytes, 256-byte aligned.
 */
size_t amq_softmax_layer_workspace_bytes(int64_t V, int64_t H, int64_t B, int k_a);
int amq_softmax_layer(const uint32_t* Wsp, const float* alpha_s, int64_t V, int64_t H, int k_w,
                      const float* bias, const float* h, int64_t B, int k_a, int T, float* logprob,
                      void* workspace, size_t workspace_bytes, void* stream);

/*
 * One whole language-model step, Eq. 6 from token to distribution: x_t = row ids[b] of the quantized
 * embedding (k_a planes: the table must be quantized with k = k_a), h_{t-1} quantized on line (k_a),
 * LSTM cell (h and c [B][H] are read and overwritten), h_t quantized again (k_as) and the output
 * layer W_s (V x H, k_ws-bit) with log-softmax -> logprob [B][V].
 *   workspace: at least amq_lm_workspace_bytes(E, H, V, B, k_a, k_as) bytes, 256-byte aligned.
 */
size_t amq_lm_workspace_bytes(int64_t E, int64_t H, int64_t V, int64_t B, int k_a, int k_as);
int amq_lm_step(const uint32_t* Ep, const float* alpha_e, int64_t vocab, int64_t E, const uint32_t* Wxp,
                const float* alpha_x, const uint32_t* Whp, const float* alpha_h, int64_t H, int k_w,
                const float* bias, const uint32_t* Wsp, const float* alpha_s, int64_t V, int k_ws,
                const float* bias_s, const int64_t* ids, float* h, float* c, int64_t B, int k_a, int k_as,
                int T, float* logprob, void* workspace, size_t workspace_bytes, void* stream);

/*
 * `steps` consecutive language-model steps in one call: ids [steps][B], logprob [steps][B][V];
 * h and c [B][H] are read as the initial state and overwritten with the final state.  Same
 * arithmetic as `steps` calls of amq_lm_step.  For B = 1 (with E, H <= 1024 and 2- or 3-bit codes)
 * the recurrence runs in one launch per 64 steps (see amq_lstm_sequence, including its residency
 * requirement and its flag word: amq_lstm_sequence_flag_offset(E, H, 1, k_a) applies to this
 * workspace too; AMQ_OK does not cover a give-up, after which the log-probabilities from the piece
 * that gave up onwards are NaN) and the output layer then takes all h_t of those steps as one batch.  For larger
 * B the recurrent halves of the steps run one after the other and the output layer takes the
 * hidden states of about 4096 / B steps at a time (the inputs are given, so only the recurrence
 * is serial: where the shape allows, the input rows are looked up one step ahead and W_x x_t is
 * formed beside the quantization of h_{t-1}, as in amq_lstm_sequence); the workspace holds those
 * hidden states, the looked-up codes of two steps and the x-side sums of one.
 *   workspace: at least amq_lm_sequence_workspace_bytes(E, H, V, B, k_a, k_as) bytes, 256-byte aligned.
 */
size_t amq_lm_sequence_workspace_bytes(int64_t E, int64_t H, int64_t V, int64_t B, int k_a, int k_as);
int amq_lm_sequence(const uint32_t* Ep, const float* alpha_e, int64_t vocab, int64_t E,
                    const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp, const float* alpha_h,
                    int64_t H, int k_w, const float* bias, const uint32_t* Wsp, const float* alpha_s,
                    int64_t V, int k_ws, const float* bias_s, const int64_t* ids, int64_t steps, float* h,
                    float* c, int64_t B, int k_a, int k_as, int T, float* logprob, void* workspace,
                    size_t workspace_bytes, void* stream);

/*
 * Scoring a given continuation (the quantity behind the perplexities of Sec. 5): the same steps as
 * amq_lm_sequence, but only the log-probability of one given word per step and batch entry is
 * returned: target_logprob[t][b] = logprob[t][b][targets[t][b]] (device, [steps][B]).  targets
 * [steps][B] (device) are row indices of W_s; an index outside [0, V) gives NaN.  Where the output
 * layer is large enough for the matrix-core kernel with several batch tiles per wave, the logits
 * are never written to memory (the kernel leaves the chosen logit and the partial log-sum-exp);
 * otherwise 64 rows at a time go through the ordinary layer.  Same arithmetic as amq_lm_sequence.
 *   workspace: at least amq_lm_sequence_score_workspace_bytes(E, H, V, B, k_a, k_as) bytes, 256-byte
 *   aligned (the flag word of the batch-1 recurrence sits at the same offset as in amq_lm_sequence).
 */
size_t amq_lm_sequence_score_workspace_bytes(int64_t E, int64_t H, int64_t V, int64_t B, int k_a, int k_as);
int amq_lm_sequence_score(const uint32_t* Ep, const float* alpha_e, int64_t vocab, int64_t E,
                          const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp, const float* alpha_h,
                          int64_t H, int k_w, const float* bias, const uint32_t* Wsp, const float* alpha_s,
                          int64_t V, int k_ws, const float* bias_s, const int64_t* ids, const int64_t* targets,
                          int64_t steps, float* h, float* c, int64_t B, int k_a, int k_as, int T,
                          float* target_logprob, void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* AMQ_H_ */
