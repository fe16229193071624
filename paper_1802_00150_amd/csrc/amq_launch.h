// Host-side launch interface between the C ABI (amq_api.hip) and the kernel files.
// Everything here is plain data plus one launch function per kernel family; argument
// checking happens in the C ABI layer before any of these are called.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace amq {

// Raises the dynamic-LDS limit of kernel `fn` to `bytes` the first time it is launched on the current
// device.  `done` is the kernel instantiation's own mask of devices already configured (thread-safe;
// devices numbered 64 and above are configured at every launch).
inline hipError_t ensure_dynamic_lds(const void* fn, int bytes, std::atomic<unsigned long long>& done) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const bool tracked = dev >= 0 && dev < 64;
  if (tracked && ((done.load(std::memory_order_acquire) >> dev) & 1ull)) return hipSuccess;
  e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e != hipSuccess) return e;
  if (tracked) done.fetch_or(1ull << dev, std::memory_order_release);
  return hipSuccess;
}

#ifdef AMQ_PHASE_TIMING
// Profiling build only: the device buffer the phase timers write to (null: timers off), set through
// the extra entry point amq_debug_set_phase_buffer of that build.
unsigned long long* phase_buffer();
#define AMQ_PHASE_MEMBER unsigned long long* phase;
#define AMQ_PHASE_ATTACH(args) (args).phase = ::amq::phase_buffer()
#define AMQ_PHASE_OF(args) (args).phase
#else
#define AMQ_PHASE_MEMBER
#define AMQ_PHASE_ATTACH(args) \
  do {                         \
  } while (0)
#define AMQ_PHASE_OF(args) nullptr
#endif

// ---- quantizer -------------------------------------------------------------------------
enum { kQuantFull = 0, kQuantLsOnly = 1, kQuantBstOnly = 2 };

struct QuantSeg {
  const float* X;    // [count][ld]
  long long ld;      // row stride in elements
  int n;             // vector length
  int count;         // number of vectors (0 = segment unused)
  uint32_t* planes;  // [k][count][wpr(n)]
  float* coef;       // [count][k]
};

// Rows of a quantized table copied out by index in the same launch (the embedding lookup of a
// language-model step): table planes [k][vocab][wpr(n)], coefficients [vocab][k].  An index
// outside [0, vocab) yields the zero vector (all plane bits 0, coefficients 0).
struct GatherSeg {
  const uint32_t* table;   // [k][vocab][wpr(n)]
  const float* table_coef; // [vocab][k]
  long long vocab;
  const long long* ids;    // [count]
  int n;
  int count;               // 0 = unused
  uint32_t* planes;        // [k][count][wpr(n)]
  float* coef;             // [count][k]
};

// Up to two groups of vectors in one launch (x_t and h_{t-1} of a recurrent step), plus an
// optional gather of already quantized rows.
struct QuantArgs {
  QuantSeg seg[2];
  int T;
  int mode;
  GatherSeg gather;
  AMQ_PHASE_MEMBER
};

hipError_t launch_quantize(const QuantArgs& a, int k, hipStream_t s);

// ---- comparison quantizer and error measure ------------------------------------------------
// Refined greedy approximation of `count` vectors X [count][ld] of length n (Sec. 2).
hipError_t launch_refined_greedy(const float* X, long long ld, int n, int count, int k, uint32_t* planes, float* coef,
                                 hipStream_t s);
// Sums of squared error and squared norm of every row, then result = {error, norm, error / norm}.
// ternary quantization as 2-bit codes with equal coefficients (Sec. 2)
hipError_t launch_ternary(const float* X, long long ld, int n, int count, int T, uint32_t* planes, float* coef,
                          hipStream_t s);
hipError_t launch_relative_mse(const float* W, long long rows, int cols, long long ld, int k, const uint32_t* planes,
                               const float* alpha, double* row_err, double* row_norm, double* result,
                               hipStream_t s);

// Reconstruction out[r][l] = sum_i +-alpha[r][i] (the binary32 code-table value of the entry's code).
hipError_t launch_dequantize(const uint32_t* planes, const float* alpha, long long rows, int cols, int k, float* out,
                             long long ld_out, hipStream_t s);
// In-place clipping of n values to [lo, hi].
hipError_t launch_clip(float* w, long long n, float lo, float hi, hipStream_t s);

// ---- binary products -------------------------------------------------------------------
struct GemmOperand {
  const uint32_t* Wp;   // [k_w][m][wpr]
  const float* alpha;   // [m][k_w]
  const uint32_t* Xp;   // [k_a][batch][wpr]
  const float* beta;    // [batch][k_a]
  int n;                // vector length of this block
};

struct GemmArgs {
  GemmOperand op;
  long long m;
  int batch;
  int k_w, k_a;
  const float* bias;   // [m] or null
  int accumulate;
  float* Y;            // [batch][m] or null
  int32_t* D;          // [batch][m][k_w][k_a] or null (test hook)
  float* lse_part;     // null, or room for lse_cap (max, sum-of-exponentials) pairs per batch entry
  int lse_cap;
  // grouped batch-1 products: strides in elements between consecutive groups (0 when groups == 1)
  int groups;
  long long g_Wp, g_alpha, g_Xp, g_beta, g_Y;
};

hipError_t launch_gemm(const GemmArgs& a, hipStream_t s);

// ---- small-batch products with weights in registers and fused epilogues --------------------
enum { kEpiStore = 0, kEpiLstm = 1, kEpiGru = 2 };
// Largest batch the small-batch kernel takes.  Where the fp4 matrix-core kernels apply (vectors of at
// most 1024 entries) they are faster from batch 5 on for a plain product and from batch 2 on for a
// fused cell step (measured, 4096 x 1024 and the 1024-unit LSTM, W2/A2 and W3/A3: plain product 3.6-4.0
// against 3.8-4.6 us at batch 4, 4.6-5.8 against 3.8-4.6 us at batch 8; LSTM step 5.2-6.6 against
// 5.9-9.0 us at batch 1, 6.8-9.2 against 5.9-9.0 us at batch 2, 29-44 against 5.5-7.5 us at batch 16);
// for longer vectors the alternative is the int8 kernel and the old limit stays.
constexpr int kBmvMaxBatch = 16;
constexpr int kBmvMaxBatchStore = 4;
constexpr int kBmvMaxBatchCell = 1;
// weight planes of one launch beyond this many bytes cannot stay in the 256 MB last-level cache between
// launches: the small-batch kernel then reads them with non-temporal loads
constexpr long long kBmvStreamingBytes = 128LL << 20;

struct BmvBlock {
  const uint32_t* Wp;   // [k_w][m][wpr(n)]
  const float* alpha;   // [m][k_w]
  const uint32_t* Xp;   // [k_a][batch][wpr(n)]
  const float* beta;    // [batch][k_a]
  int n;
};

struct BmvArgs {
  BmvBlock blk[2];      // x block, h block (store mode uses blk[0] only)
  long long m;          // rows per plane (4H for the LSTM, 3H for the GRU)
  long long H;          // hidden units (cell modes)
  int batch;
  const float* bias0;   // store: [m]; LSTM: [4H]; GRU: bias_x [3H]   (nullable)
  const float* bias1;   // GRU: bias_h [3H] (nullable)
  int accumulate;       // store mode
  float* Y;             // store mode: [batch][m]
  int32_t* D;           // store mode, matrix-core kernel only: [batch][m][k_w][k_a] integer dots (nullable)
  const float* c_prev;  // LSTM
  const float* h_prev;  // GRU
  float* h_out;
  float* c_out;
  float* hs_out;        // nullable second destination of h_t: LSTM; GRU in the paired kernel and its split forms
  float* lse_part;      // store mode, nullable: per batch entry and slot a (max, sum exp(y - max)) pair over
                        // the outputs one wave produced, [batch][lse_slots][2]
  int lse_slots;        // filled by the launcher: slots per batch entry
  int lse_cap;          // slots per batch entry the buffer has room for
  const long long* tgt; // several-tiles store kernel only, nullable: one output row index per batch entry ...
  float* tgt_out;       // ... whose output value is also written here, [batch] (Y may then be null)
  int lg;               // filled by launch_bmv
  int streaming;        // filled by launch_bmv: planes are read once, load them non-temporal
  int groups;           // small-batch kernel: independent products / cells in one launch (1 otherwise)
  // strides in elements between consecutive groups: operands of the x block, of the h block (LSTM
  // mode), outputs of store mode, and state vectors (c_prev, h_out, c_out, hs_out) of LSTM mode
  long long g_Wp, g_alpha, g_Xp, g_beta, g_Y;
  long long g_Wp1, g_alpha1, g_Xp1, g_beta1, g_state;
  AMQ_PHASE_MEMBER
};

// Most (max, sum) slots per batch entry worth merging afterwards; a launch that would need more
// (or more than the buffer's lse_cap) leaves lse_part untouched and reports 0 slots.
constexpr int kLseMaxSlots = 8192;

// true if the register-resident kernel can take these vector lengths / batch
bool bmv_supported(int n0, int n1, int k_a, long long batch, int epi);
// lse_slots (nullable) receives the number of slots written per batch entry when a.lse_part is set
hipError_t launch_bmv(BmvArgs a, int k_w, int k_a, int epi, hipStream_t s, int* lse_slots = nullptr);

// ---- batched products on the matrix cores (int8 MFMA on expanded codes), same epilogues ------
bool mfma_supported(long long batch);
hipError_t launch_mfma(const BmvArgs& a, int k_w, int k_a, int epi, hipStream_t s);
// fp4 matrix-core kernel for vectors of at most 1024 entries (the fast path)
bool mfma4_supported(const BmvArgs& a, int k_w, int epi);
hipError_t launch_mfma4(BmvArgs a, int k_w, int k_a, int epi, hipStream_t s, int* lse_slots = nullptr);
// the same instruction with several batch tiles per wave: plain products with many rows and
// at least 32 columns (store mode only)
bool mfma4w_supported(const BmvArgs& a, int k_w, int k_a);
hipError_t launch_mfma4w(const BmvArgs& a, int k_w, int k_a, hipStream_t s, int* lse_slots = nullptr);
// the recurrent steps with both operands loaded straight into registers in sign form and the x / h
// blocks on paired waves (batches of 17 and more while the row-block x tile tasks are few)
bool mfma4_pair_supported(const BmvArgs& a, int k_w, int k_a, int epi);
hipError_t launch_mfma4_pair(const BmvArgs& a, int k_w, int k_a, int epi, hipStream_t s);
// and the recurrent steps in the same work split, for batches of 128 and more
bool mfma4w_cell_supported(const BmvArgs& a, int k_w, int k_a, int epi);
hipError_t launch_mfma4w_cell(const BmvArgs& a, int k_w, int k_a, int epi, hipStream_t s);

// ---- output layer -----------------------------------------------------------------------
// out[b][v] = Y[b][v] - log(sum_u exp(Y[b][u])); out may alias Y.
hipError_t launch_log_softmax(const float* Y, long long B, long long V, float* out, hipStream_t s);
// The same when a product kernel has already reduced its outputs to `slots` (max, sum) pairs per row.
hipError_t launch_log_softmax_finish(const float* Y, long long B, long long V, const float* part, int slots,
                                     float* out, hipStream_t s);
// out[b] = value[b] - log(sum_u exp(Y[b][u])) from the (max, sum) pairs alone; an index outside [0, V)
// gives NaN
hipError_t launch_score_finish(const float* value, const long long* index, long long B, long long V, const float* part,
                               int slots, float* out, hipStream_t s);
// out[b] = logprob[b][index[b]] (NaN for an index outside [0, V))
hipError_t launch_gather_columns(const float* logprob, long long B, long long V, const long long* index, float* out,
                                 hipStream_t s);

// ---- whole batch-1 LSTM sequences in one launch spread over the chip (weights resident in
// registers; the workgroups exchange h_t as tagged entries, one grid barrier per launch) ------
constexpr int kSeqGMaxGrid = 256;   // workgroups: one per compute unit, all resident at once
constexpr int kSeqGMaxSteps = 64;   // time steps per launch (size of the table of input codes)
struct SeqGArgs {
  const uint32_t* Wxp;  // [k_w][4H][wpr(I)]
  const float* ax;      // [4H][k_w]
  const uint32_t* Whp;  // [k_w][4H][wpr(H)]
  const float* ah;      // [4H][k_w]
  int I, H;
  const float* bias;    // [4H] or null
  const float* xs;      // [steps][I], or null: xq / xbeta already hold the codes of the inputs
  int steps;            // at most kSeqGMaxSteps
  float* h;             // [H] in: h_0, out: h_steps
  float* c;             // [H] in: c_0, out: c_steps
  float* hs;            // [steps][H] or null
  int T;
  int lg;               // filled by launch_lstm_seqg
  // scratch in global memory (the caller's workspace)
  unsigned* sync;       // give-up flag (left non-zero if the launch was abandoned), then kSeqGMaxGrid arrival bytes
  unsigned long long* hbuf;  // [2][H]: h_t as published by the grid, {value, step tag} pairs, double-buffered
  uint32_t* xq;         // [k_a][steps][wpr(I)]: codes of the inputs (operand layout)
  float* xbeta;         // [steps][k_a]: their coefficients
  int first_piece;      // non-zero: also clear the give-up flag (once per API call; a later piece of the
                        // same call must see a flag an earlier piece raised)
  unsigned spin_limit;  // filled by launch_lstm_seqg: polls of a wait before it gives up
};
bool lstm_seqg_supported(long long I, long long H, long long B, int k_w, int k_a);
hipError_t launch_lstm_seqg(SeqGArgs a, int k_w, int k_a, hipStream_t s);
// Polls before a wait of the sequence kernel gives up (0 restores the default).  Tests of the failure
// path set it to 1, which makes the first wait that is not satisfied at once give up.
void set_seqg_spin_limit(unsigned polls);
// After a launch of the sequence kernel and whatever consumed its hs: if the give-up flag is set,
// overwrite out[0 .. count) with NaN (results computed from an incomplete recurrence must not look valid).
hipError_t launch_seqg_poison(const unsigned* sync, float* out, long long count, hipStream_t s);

// ---- the recurrent step of a sequence with given inputs, cut along the operand blocks ----------
// Front launch: quantizes the vectors of q (seg[0] = h_{t-1}, seg[1] = a later x, count 0 for none) and of
// q2 (nullable; more inputs, at the first step), and forms the x-side product x (nullable; operand block 0
// of *x: codes from an earlier front launch; x->Y receives the sums as [batch][H][4]).  Back launch:
// h-side products of a (operand block 1), plus the x-side sums in a.Y, then the cell.  Same shapes as the
// paired one-tile kernel, k_w and k_a at most 3.
bool step_split_supported(const BmvArgs& b, int k_w, int k_a, int epi);
hipError_t launch_step_front(const QuantArgs& q, const QuantArgs* q2, const BmvArgs* x, int k_w, int k_a, int epi,
                             hipStream_t s);
hipError_t launch_step_back(BmvArgs a, int k_w, int k_a, int epi, hipStream_t s);

// ---- bandwidth yardstick ------------------------------------------------------------------
// Reads `bytes` (a multiple of 16) once with 16-byte loads over kStreamReadBlocks workgroups and leaves
// an xor checksum per workgroup in sink [kStreamReadBlocks].
constexpr int kStreamReadBlocks = 4096;
hipError_t launch_stream_read(const void* buf, size_t bytes, unsigned long long* sink, hipStream_t s);

// ---- cells -----------------------------------------------------------------------------
// pre-activations -> new state, Eq. 6 (LSTM) and the reset-after GRU
hipError_t launch_lstm_pointwise(const float* pre /*[B][4H]*/, const float* c_prev, float* h_out,
                                 float* c_out, float* hs_out /*nullable*/, long long B, long long H,
                                 hipStream_t s);
hipError_t launch_gru_pointwise(const float* pre_x /*[B][3H]*/, const float* pre_h, const float* h_prev,
                                float* h_out, long long B, long long H, hipStream_t s);
// GRU with the reset gate applied before the candidate's hidden-side product: g = r * h_prev, then
// (with pre_g = Wh q(g) + bias_h) the rest of the cell
hipError_t launch_gru_rb_reset(const float* pre_x, const float* pre_h, const float* h_prev, float* g_out, long long B,
                               long long H, hipStream_t s);
hipError_t launch_gru_rb_final(const float* pre_x, const float* pre_h, const float* pre_g, const float* h_prev,
                               float* h_out, long long B, long long H, hipStream_t s);

}  // namespace amq
