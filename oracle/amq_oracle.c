/*
 * amq_oracle.c -- plain CPU oracle for alternating multi-bit quantization and
 * the quantized LSTM / GRU inference step built on it.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It exists so that the GPU
 * library can be checked against something written directly from the paper.
 * Only the tests, the smoke check and the benchmark's cpu_baseline leg may
 * call it.  It shares no code, header, table or helper with the GPU library.
 *
 * Style: scalar loops in the paper's order and notation, no blocking, no
 * fusion, no intrinsics.  Precision rule (one place, applies everywhere):
 *   - every quantity the method stores (w, residual r, alpha, the code table
 *     v, the midpoints, outputs y / h / c) is IEEE binary32;
 *   - a single operation on stored values (r - alpha, v sums, 0.5*(a+b)) is
 *     done in binary32, so that the comparison "w >= midpoint" which decides a
 *     binary code is taken in binary32 on both sides of a parity test;
 *   - every reduction (sum |r|, B^T w, the error, the coefficient epilogue,
 *     gate pre-activations), the k x k solve and the transcendental functions
 *     are done in binary64 and rounded to binary32 once.
 *
 * Pinned (tests/test_oracle_*.py): greedy against Eq. 4 closed forms on
 * Gaussian data; k = 1 closed form; BST against brute-force nearest code;
 * Fig. 1 boundaries; k = 2 closed form; LS against a library least-squares
 * routine; non-increasing error over the half-steps of Alg. 2; binary dots
 * against an integer matrix product on unpacked +-1 codes; GEMM and the two
 * cells against dense fp64 products of the de-quantized operands; the
 * embedding lookup against quantizing the looked-up row; the log-softmax
 * against a library routine, the two-class closed form and normalisation;
 * the output layer against a dense fp64 layer on de-quantized operands;
 * the reset-before GRU against a dense fp64 cell and against the reset-after
 * cell when the reset gate is saturated; the trailing-least-squares variant against a library least-squares routine;
 * the reconstruction against the code table and a dense product; refined
 * greedy against a library least-squares routine stage by stage; the
 * relative error against a norm computed by a library; the operation-count
 * model of Sec. 4.
 * Parity unpinned: nothing in this file.  (Trained-model accuracy tables are
 * outside what this oracle computes.)
 *
 * Build: gcc -O3 -ffp-contract=off -fopenmp -shared -fPIC (see oracle/build.py).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_MAX_K 4

static int g_threads = 1;

/* Number of host threads the row- / batch-parallel entry points may use. */
void amq_oracle_set_threads(int t) { g_threads = t < 1 ? 1 : t; }

int amq_oracle_get_threads(void) {
#ifdef _OPENMP
  int mx = omp_get_max_threads();
  return g_threads < mx ? g_threads : mx;
#else
  return 1;
#endif
}

/* Packing convention of the exchange format: 32-bit words per row per plane,
 * rows padded to a multiple of 128 entries (16 bytes). */
int64_t amq_oracle_wpr(int64_t n) { return 4 * ((n + 127) / 128); }

/* sign(x) = +1 iff x >= 0 (so -0.0 maps to +1), as a 0/1 code.  Matches the
 * ">=" of Alg. 1. */
static uint8_t sign_code(float x) { return x >= 0.0f ? 1 : 0; }

static float code_value(uint8_t c) { return c ? 1.0f : -1.0f; }

/* ------------------------------------------------------------------ *
 * Greedy approximation, Eq. 3-4: r_0 = w; alpha_i = ||r_{i-1}||_1 / n,
 * b_i = sign(r_{i-1}), r_i = r_{i-1} - alpha_i b_i.
 * code is [k][n] with entries 0 (-1) / 1 (+1).
 * ------------------------------------------------------------------ */
void amq_oracle_greedy(const float* w, int64_t n, int k, uint8_t* code, float* alpha) {
  float* r = (float*)malloc(sizeof(float) * (size_t)n);
  memcpy(r, w, sizeof(float) * (size_t)n);
  for (int i = 0; i < k; ++i) {
    double l1 = 0.0;
    for (int64_t l = 0; l < n; ++l) l1 += fabs((double)r[l]);
    alpha[i] = (float)(l1 / (double)n);
    for (int64_t l = 0; l < n; ++l) {
      uint8_t b = sign_code(r[l]);
      code[(size_t)i * n + l] = b;
      r[l] = r[l] - alpha[i] * code_value(b); /* binary32; the product is exact */
    }
  }
  free(r);
}

/* Exact determinant of a k x k integer matrix by cofactor expansion. */
static __int128 int_det(const int64_t* G, int k, int stride) {
  if (k == 1) return (__int128)G[0];
  __int128 d = 0;
  int64_t M[ORACLE_MAX_K * ORACLE_MAX_K];
  for (int c = 0; c < k; ++c) {
    for (int i = 1; i < k; ++i) {
      int cc = 0;
      for (int j = 0; j < k; ++j) {
        if (j == c) continue;
        M[(i - 1) * (k - 1) + cc] = G[i * stride + j];
        ++cc;
      }
    }
    __int128 minor = int_det(M, k - 1, k - 1);
    d += ((c & 1) ? -1 : 1) * (__int128)G[c] * minor;
  }
  return d;
}

/* ------------------------------------------------------------------ *
 * Least-squares coefficients, Eq. 5: alpha = (B^T B)^{-1} B^T w with
 * B = [b_1 .. b_k].  B^T B is an integer matrix (entries n - 2 * #disagree).
 * If it is singular (exact integer test) the coefficients are left as they
 * are and 0 is returned; otherwise alpha is overwritten and 1 is returned.
 * The solve is Gaussian elimination with partial pivoting in binary64.
 * ------------------------------------------------------------------ */
int amq_oracle_ls(const float* w, int64_t n, int k, const uint8_t* code, float* alpha) {
  int64_t G[ORACLE_MAX_K * ORACLE_MAX_K];
  double q[ORACLE_MAX_K];
  for (int i = 0; i < k; ++i) {
    for (int j = 0; j < k; ++j) {
      int64_t s = 0;
      for (int64_t l = 0; l < n; ++l) {
        int bi = code[(size_t)i * n + l] ? 1 : -1;
        int bj = code[(size_t)j * n + l] ? 1 : -1;
        s += bi * bj;
      }
      G[i * k + j] = s;
    }
    double acc = 0.0;
    for (int64_t l = 0; l < n; ++l)
      acc += code[(size_t)i * n + l] ? (double)w[l] : -(double)w[l];
    q[i] = acc;
  }
  if (int_det(G, k, k) == 0) return 0;

  double A[ORACLE_MAX_K][ORACLE_MAX_K + 1];
  for (int i = 0; i < k; ++i) {
    for (int j = 0; j < k; ++j) A[i][j] = (double)G[i * k + j];
    A[i][k] = q[i];
  }
  for (int c = 0; c < k; ++c) {
    int p = c;
    for (int i = c + 1; i < k; ++i)
      if (fabs(A[i][c]) > fabs(A[p][c])) p = i;
    if (p != c)
      for (int j = 0; j <= k; ++j) { double t = A[c][j]; A[c][j] = A[p][j]; A[p][j] = t; }
    for (int i = c + 1; i < k; ++i) {
      double f = A[i][c] / A[c][c];
      for (int j = c; j <= k; ++j) A[i][j] -= f * A[c][j];
    }
  }
  double x[ORACLE_MAX_K];
  for (int i = k - 1; i >= 0; --i) {
    double s = A[i][k];
    for (int j = i + 1; j < k; ++j) s -= A[i][j] * x[j];
    x[i] = s / A[i][i];
  }
  for (int i = 0; i < k; ++i) alpha[i] = (float)x[i];
  return 1;
}

/* ------------------------------------------------------------------ *
 * Code table of Alg. 2 ("construct v in ascending order"): all 2^k values
 * s_1 alpha_1 + ... + s_k alpha_k.  Pattern p in [0, 2^k) has s_i = +1 iff bit
 * (k - i) of p is set, so that for alpha_1 >= ... >= alpha_k >= 0 the natural
 * order of p is already ascending.  Values are summed left to right in
 * binary32.  Pairs (value, p) are sorted ascending by value, ties by p.
 * mid[j] = 0.5 * (v[j] + v[j+1]) in binary32, j = 0 .. 2^k - 2.
 * ------------------------------------------------------------------ */
void amq_oracle_code_table(const float* alpha, int k, float* v, int32_t* pattern, float* mid) {
  int m = 1 << k;
  for (int p = 0; p < m; ++p) {
    float s = 0.0f;
    for (int i = 1; i <= k; ++i) {
      float term = ((p >> (k - i)) & 1) ? alpha[i - 1] : -alpha[i - 1];
      s = (i == 1) ? term : s + term;
    }
    v[p] = s;
    pattern[p] = p;
  }
  /* insertion sort: stable, so equal values keep ascending p */
  for (int a = 1; a < m; ++a) {
    float va = v[a];
    int32_t pa = pattern[a];
    int b = a - 1;
    while (b >= 0 && v[b] > va) {
      v[b + 1] = v[b];
      pattern[b + 1] = pattern[b];
      --b;
    }
    v[b + 1] = va;
    pattern[b + 1] = pa;
  }
  for (int j = 0; j + 1 < m; ++j) mid[j] = 0.5f * (v[j] + v[j + 1]);
}

/* Alg. 1 for one entry: walk the sorted table, halving the feasible range,
 * going to the upper half iff w >= midpoint of the two codes at the split.
 * Returns the position in the sorted table. */
static int bst_walk(float w, const float* mid, int lo, int hi) {
  int len = hi - lo;
  if (len == 1) return lo;
  int half = lo + len / 2;
  if (w >= mid[half - 1]) return bst_walk(w, mid, half, hi);
  return bst_walk(w, mid, lo, half);
}

/* ------------------------------------------------------------------ *
 * Binary codes with the coefficients fixed (Alg. 1 applied to every entry).
 * ------------------------------------------------------------------ */
void amq_oracle_bst(const float* w, int64_t n, int k, const float* alpha, uint8_t* code) {
  float v[1 << ORACLE_MAX_K], mid[1 << ORACLE_MAX_K];
  int32_t pattern[1 << ORACLE_MAX_K];
  amq_oracle_code_table(alpha, k, v, pattern, mid);
  for (int64_t l = 0; l < n; ++l) {
    int pos = bst_walk(w[l], mid, 0, 1 << k);
    int p = pattern[pos];
    for (int i = 1; i <= k; ++i) code[(size_t)(i - 1) * n + l] = (uint8_t)((p >> (k - i)) & 1);
  }
}

/* Objective of Eq. 2 in binary64: || w - sum_i alpha_i b_i ||^2. */
double amq_oracle_error(const float* w, int64_t n, int k, const uint8_t* code, const float* alpha) {
  double e = 0.0;
  for (int64_t l = 0; l < n; ++l) {
    double rec = 0.0;
    for (int i = 0; i < k; ++i) rec += code[(size_t)i * n + l] ? (double)alpha[i] : -(double)alpha[i];
    double d = (double)w[l] - rec;
    e += d * d;
  }
  return e;
}

/* ------------------------------------------------------------------ *
 * Alg. 2: greedy initialisation, then T times { Eq. 5; code table; Alg. 1 }.
 * No trailing least-squares step: the returned alpha are those used by the
 * last code assignment.  trace (nullable) receives 1 + 2T objective values:
 * after greedy, then after each coefficient update and each code update.
 * ------------------------------------------------------------------ */
void amq_oracle_quantize(const float* w, int64_t n, int k, int T, uint8_t* code, float* alpha,
                         double* trace) {
  amq_oracle_greedy(w, n, k, code, alpha);
  if (trace) trace[0] = amq_oracle_error(w, n, k, code, alpha);
  for (int it = 0; it < T; ++it) {
    amq_oracle_ls(w, n, k, code, alpha);
    if (trace) trace[1 + 2 * it] = amq_oracle_error(w, n, k, code, alpha);
    amq_oracle_bst(w, n, k, alpha, code);
    if (trace) trace[2 + 2 * it] = amq_oracle_error(w, n, k, code, alpha);
  }
}

/* Pack one plane of n 0/1 codes: entry l -> word l / 32, bit l % 32, bit 1
 * means +1.  All wpr(n) words are written; bits past n are 0. */
void amq_oracle_pack(const uint8_t* code, int64_t n, uint32_t* words) {
  int64_t wpr = amq_oracle_wpr(n);
  for (int64_t j = 0; j < wpr; ++j) words[j] = 0u;
  for (int64_t l = 0; l < n; ++l)
    if (code[l]) words[l / 32] |= (uint32_t)1 << (l % 32);
}

static int unpack_bit(const uint32_t* words, int64_t l) { return (int)((words[l / 32] >> (l % 32)) & 1u); }

/* ------------------------------------------------------------------ *
 * Row-wise quantization of a matrix (Sec. 4: one coefficient set per row), also used for a
 * batch of activation vectors.  W is rows x cols with leading dimension ld.
 * planes: [k][rows][wpr] words, alpha: [rows][k].
 * ------------------------------------------------------------------ */
void amq_oracle_quantize_rows(const float* W, int64_t rows, int64_t cols, int64_t ld, int k, int T,
                              uint32_t* planes, float* alpha) {
  int64_t wpr = amq_oracle_wpr(cols);
#ifdef _OPENMP
#pragma omp parallel for num_threads(amq_oracle_get_threads()) schedule(static)
#endif
  for (int64_t r = 0; r < rows; ++r) {
    uint8_t* code = (uint8_t*)malloc((size_t)k * (size_t)cols);
    float a[ORACLE_MAX_K];
    amq_oracle_quantize(W + r * ld, cols, k, T, code, a, NULL);
    for (int i = 0; i < k; ++i) {
      amq_oracle_pack(code + (size_t)i * cols, cols, planes + ((size_t)i * rows + r) * wpr);
      alpha[r * k + i] = a[i];
    }
    free(code);
  }
}

/* ------------------------------------------------------------------ *
 * Binary inner products (App. A): for every batch entry b, row r, weight
 * plane i and activation plane j,
 *   D[b][r][i][j] = sum_l Bw_i[r][l] * c_j[b][l]   with entries in {-1,+1}.
 * Wp: [k_w][m][wpr], Xp: [k_a][batch][wpr], D: [batch][m][k_w][k_a].
 * ------------------------------------------------------------------ */
void amq_oracle_binary_dots(const uint32_t* Wp, int64_t m, int64_t n, int k_w, const uint32_t* Xp,
                            int64_t batch, int k_a, int32_t* D) {
  int64_t wpr = amq_oracle_wpr(n);
  /* activation codes unpacked once to +-1 */
  int8_t* xs = (int8_t*)malloc((size_t)k_a * (size_t)batch * (size_t)n);
  for (int j = 0; j < k_a; ++j)
    for (int64_t b = 0; b < batch; ++b)
      for (int64_t l = 0; l < n; ++l)
        xs[((size_t)j * batch + b) * n + l] =
            unpack_bit(Xp + ((size_t)j * batch + b) * wpr, l) ? 1 : -1;
#ifdef _OPENMP
#pragma omp parallel for num_threads(amq_oracle_get_threads()) schedule(static)
#endif
  for (int64_t r = 0; r < m; ++r) {
    int8_t* ws = (int8_t*)malloc((size_t)n);
    for (int i = 0; i < k_w; ++i) {
      for (int64_t l = 0; l < n; ++l) ws[l] = unpack_bit(Wp + ((size_t)i * m + r) * wpr, l) ? 1 : -1;
      for (int64_t b = 0; b < batch; ++b) {
        for (int j = 0; j < k_a; ++j) {
          const int8_t* x = xs + ((size_t)j * batch + b) * n;
          int32_t s = 0;
          for (int64_t l = 0; l < n; ++l) s += (int32_t)ws[l] * (int32_t)x[l];
          D[(((size_t)b * m + r) * k_w + i) * k_a + j] = s;
        }
      }
    }
    free(ws);
  }
  free(xs);
}

/* ------------------------------------------------------------------ *
 * Quantized matrix product (Sec. 4, Fig. 3 left): binary products first,
 * then the coefficients:
 *   Y[b][r] = (accumulate ? Y[b][r] : 0) + bias[r]
 *             + sum_i alpha[r][i] * sum_j beta[b][j] * D[b][r][i][j]
 * evaluated in binary64 and rounded once.  bias may be NULL.
 * ------------------------------------------------------------------ */
void amq_oracle_binary_gemm(const uint32_t* Wp, const float* alpha, int64_t m, int64_t n, int k_w,
                            const uint32_t* Xp, const float* beta, int64_t batch, int k_a,
                            const float* bias, int accumulate, float* Y) {
  int32_t* D = (int32_t*)malloc(sizeof(int32_t) * (size_t)batch * (size_t)m * (size_t)(k_w * k_a));
  amq_oracle_binary_dots(Wp, m, n, k_w, Xp, batch, k_a, D);
  for (int64_t b = 0; b < batch; ++b)
    for (int64_t r = 0; r < m; ++r) {
      double y = accumulate ? (double)Y[b * m + r] : 0.0;
      if (bias) y += (double)bias[r];
      for (int i = 0; i < k_w; ++i) {
        double inner = 0.0;
        for (int j = 0; j < k_a; ++j)
          inner += (double)beta[b * k_a + j] * (double)D[(((size_t)b * m + r) * k_w + i) * k_a + j];
        y += (double)alpha[r * k_w + i] * inner;
      }
      Y[b * m + r] = (float)y;
    }
  free(D);
}

/* Pre-activations a[b][r] = bias[r] + quantized product on operands that are
 * already quantized, kept in binary64. */
static void preact_packed(const uint32_t* Wp, const float* alpha, int64_t m, int64_t n, int k_w,
                          const uint32_t* Xp, const float* beta, int64_t batch, int k_a,
                          const float* bias, double* a) {
  int32_t* D = (int32_t*)malloc(sizeof(int32_t) * (size_t)batch * (size_t)m * (size_t)(k_w * k_a));
  amq_oracle_binary_dots(Wp, m, n, k_w, Xp, batch, k_a, D);
  for (int64_t b = 0; b < batch; ++b)
    for (int64_t r = 0; r < m; ++r) {
      double y = bias ? (double)bias[r] : 0.0;
      for (int i = 0; i < k_w; ++i) {
        double inner = 0.0;
        for (int j = 0; j < k_a; ++j)
          inner += (double)beta[b * k_a + j] * (double)D[(((size_t)b * m + r) * k_w + i) * k_a + j];
        y += (double)alpha[r * k_w + i] * inner;
      }
      a[b * m + r] = y;
    }
  free(D);
}

/* The same with the dense operand X quantized on line first (k_a bits, T cycles). */
static void preact(const uint32_t* Wp, const float* alpha, int64_t m, int64_t n, int k_w,
                   const float* X, int64_t batch, int k_a, int T, const float* bias, double* a) {
  int64_t wpr = amq_oracle_wpr(n);
  uint32_t* Xp = (uint32_t*)malloc(sizeof(uint32_t) * (size_t)k_a * (size_t)batch * (size_t)wpr);
  float* beta = (float*)malloc(sizeof(float) * (size_t)batch * (size_t)k_a);
  amq_oracle_quantize_rows(X, batch, n, n, k_a, T, Xp, beta);
  preact_packed(Wp, alpha, m, n, k_w, Xp, beta, batch, k_a, bias, a);
  free(beta);
  free(Xp);
}

static double sigmoid(double a) { return 1.0 / (1.0 + exp(-a)); }

/* The pointwise part of Eq. 6 on binary64 pre-activations ax + ah. */
static void lstm_cell(const double* ax, const double* ah, int64_t H, int64_t B, const float* c_prev,
                      float* h_out, float* c_out) {
  int64_t m = 4 * H;
  for (int64_t b = 0; b < B; ++b)
    for (int64_t u = 0; u < H; ++u) {
      double gi = sigmoid(ax[b * m + u] + ah[b * m + u]);
      double gf = sigmoid(ax[b * m + H + u] + ah[b * m + H + u]);
      double go = sigmoid(ax[b * m + 2 * H + u] + ah[b * m + 2 * H + u]);
      double gg = tanh(ax[b * m + 3 * H + u] + ah[b * m + 3 * H + u]);
      double c = gf * (double)c_prev[b * H + u] + gi * gg;
      double h = go * tanh(c);
      c_out[b * H + u] = (float)c;
      h_out[b * H + u] = (float)h;
    }
}

/* ------------------------------------------------------------------ *
 * One quantized LSTM step, Eq. 6.  Wx is 4H x I, Wh is 4H x H, each row-wise
 * k_w-bit (planes + alpha); gate row blocks in the paper's order i, f, o, g;
 * sigmoid for i, f, o and tanh for g.  x_t and h_{t-1} are quantized on line
 * to k_a bits with T alternating cycles, each vector on its own.  bias is
 * the sum b_i + b_h, [4H], nullable.  State h, c is carried in binary32.
 * ------------------------------------------------------------------ */
void amq_oracle_lstm_step(const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp,
                          const float* alpha_h, int64_t I, int64_t H, int k_w, const float* bias,
                          const float* x, const float* h_prev, const float* c_prev, int64_t B,
                          int k_a, int T, float* h_out, float* c_out) {
  int64_t m = 4 * H;
  double* ax = (double*)malloc(sizeof(double) * (size_t)B * (size_t)m);
  double* ah = (double*)malloc(sizeof(double) * (size_t)B * (size_t)m);
  preact(Wxp, alpha_x, m, I, k_w, x, B, k_a, T, bias, ax);
  preact(Whp, alpha_h, m, H, k_w, h_prev, B, k_a, T, NULL, ah);
  lstm_cell(ax, ah, H, B, c_prev, h_out, c_out);
  free(ax);
  free(ah);
}

/* ------------------------------------------------------------------ *
 * Embedding lookup (Eq. 6, first line, with the one-hot input of a language
 * model; Sec. 4): W_e x_t is row id of the embedding matrix, and with every
 * row of W_e quantized on its own off line that row is a finished k-bit
 * quantization.
 * Ep: [k][vocab][wpr(n)], alpha_e: [vocab][k]  ->  Xp: [k][B][wpr], beta: [B][k].
 * ------------------------------------------------------------------ */
void amq_oracle_embedding_lookup(const uint32_t* Ep, const float* alpha_e, int64_t vocab, int64_t n,
                                 int k, const int64_t* ids, int64_t B, uint32_t* Xp, float* beta) {
  int64_t wpr = amq_oracle_wpr(n);
  for (int64_t b = 0; b < B; ++b) {
    int64_t id = ids[b];
    for (int i = 0; i < k; ++i) {
      for (int64_t w = 0; w < wpr; ++w)
        Xp[((size_t)i * B + b) * wpr + w] = Ep[((size_t)i * vocab + id) * wpr + w];
      beta[b * k + i] = alpha_e[id * k + i];
    }
  }
}

/* ------------------------------------------------------------------ *
 * The LSTM step of Eq. 6 with x_t arriving already quantized (packed planes
 * Xp [k_a][B][wpr(I)] and coefficients beta_x [B][k_a], e.g. looked up in a
 * quantized embedding); h_{t-1} is quantized on line as before.
 * ------------------------------------------------------------------ */
void amq_oracle_lstm_step_xq(const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp,
                             const float* alpha_h, int64_t I, int64_t H, int k_w, const float* bias,
                             const uint32_t* Xp, const float* beta_x, const float* h_prev,
                             const float* c_prev, int64_t B, int k_a, int T, float* h_out,
                             float* c_out) {
  int64_t m = 4 * H;
  double* ax = (double*)malloc(sizeof(double) * (size_t)B * (size_t)m);
  double* ah = (double*)malloc(sizeof(double) * (size_t)B * (size_t)m);
  preact_packed(Wxp, alpha_x, m, I, k_w, Xp, beta_x, B, k_a, bias, ax);
  preact(Whp, alpha_h, m, H, k_w, h_prev, B, k_a, T, NULL, ah);
  lstm_cell(ax, ah, H, B, c_prev, h_out, c_out);
  free(ax);
  free(ah);
}

/* ------------------------------------------------------------------ *
 * Logarithm of the softmax of Eq. 6 (last line), for every row:
 *   out[b][v] = Y[b][v] - log(sum_u exp(Y[b][u])),
 * evaluated in binary64 with the row maximum taken out of the exponent, and
 * rounded once.
 * ------------------------------------------------------------------ */
void amq_oracle_log_softmax(const float* Y, int64_t B, int64_t V, float* out) {
  for (int64_t b = 0; b < B; ++b) {
    const float* y = Y + (size_t)b * V;
    double mx = (double)y[0];
    for (int64_t v = 1; v < V; ++v)
      if ((double)y[v] > mx) mx = (double)y[v];
    double s = 0.0;
    for (int64_t v = 0; v < V; ++v) s += exp((double)y[v] - mx);
    double lse = mx + log(s);
    for (int64_t v = 0; v < V; ++v) out[(size_t)b * V + v] = (float)((double)y[v] - lse);
  }
}

/* ------------------------------------------------------------------ *
 * Output layer of Eq. 6: y_t = softmax(W_s h_t + b_s) with W_s (V x H)
 * row-wise k_w-bit and h_t quantized on line to k_a bits (T cycles).  The
 * logits are stored values (binary32); the log-probabilities are formed from
 * the stored logits.  logits may be NULL.
 * ------------------------------------------------------------------ */
void amq_oracle_softmax_layer(const uint32_t* Wsp, const float* alpha_s, int64_t V, int64_t H,
                              int k_w, const float* bias, const float* h, int64_t B, int k_a, int T,
                              float* logits, float* logprob) {
  double* a = (double*)malloc(sizeof(double) * (size_t)B * (size_t)V);
  float* y = logits ? logits : (float*)malloc(sizeof(float) * (size_t)B * (size_t)V);
  preact(Wsp, alpha_s, V, H, k_w, h, B, k_a, T, bias, a);
  for (size_t e = 0; e < (size_t)B * (size_t)V; ++e) y[e] = (float)a[e];
  amq_oracle_log_softmax(y, B, V, logprob);
  if (!logits) free(y);
  free(a);
}

/* ------------------------------------------------------------------ *
 * One quantized GRU step.  The paper evaluates GRUs but prints no equations;
 * this is the textbook cell in the form where the reset gate multiplies the
 * hidden-side product of the candidate, so that one quantization of h_{t-1}
 * serves all three gates:
 *   r = sigmoid(ax_r + ah_r), z = sigmoid(ax_z + ah_z),
 *   n = tanh(ax_n + r * ah_n), h = (1 - z) * n + z * h_prev,
 * with ax = Wx x + bias_x, ah = Wh h_prev + bias_h, row blocks r, z, n.
 * ------------------------------------------------------------------ */
void amq_oracle_gru_step(const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp,
                         const float* alpha_h, int64_t I, int64_t H, int k_w, const float* bias_x,
                         const float* bias_h, const float* x, const float* h_prev, int64_t B,
                         int k_a, int T, float* h_out) {
  int64_t m = 3 * H;
  double* ax = (double*)malloc(sizeof(double) * (size_t)B * (size_t)m);
  double* ah = (double*)malloc(sizeof(double) * (size_t)B * (size_t)m);
  preact(Wxp, alpha_x, m, I, k_w, x, B, k_a, T, bias_x, ax);
  preact(Whp, alpha_h, m, H, k_w, h_prev, B, k_a, T, bias_h, ah);
  for (int64_t b = 0; b < B; ++b)
    for (int64_t u = 0; u < H; ++u) {
      double r = sigmoid(ax[b * m + u] + ah[b * m + u]);
      double z = sigmoid(ax[b * m + H + u] + ah[b * m + H + u]);
      double nn = tanh(ax[b * m + 2 * H + u] + r * ah[b * m + 2 * H + u]);
      double h = (1.0 - z) * nn + z * (double)h_prev[b * H + u];
      h_out[b * H + u] = (float)h;
    }
  free(ax);
  free(ah);
}

/* ------------------------------------------------------------------ *
 * GRU step in the original form of the cell, where the reset gate multiplies
 * the previous state before the candidate's hidden-side product:
 *   r = sigmoid(ax_r + ah_r), z = sigmoid(ax_z + ah_z),
 *   n = tanh(ax_n + (Wh_n q(r * h_prev) + bias_h_n)),  h = (1 - z) * n + z * h_prev,
 * with ax = Wx q(x) + bias_x, ah = Wh q(h_prev) + bias_h (rows r, z), q = on-line
 * quantization (k_a bits, T cycles).  r * h_prev is a stored binary32 vector
 * and is quantized on line like any other activation: a second quantization
 * and a second, dependent product per step.
 * g_in (nullable): use this r * h_prev instead of computing it (staged checks);
 * g_out (nullable): receives the r * h_prev that was used.
 * ------------------------------------------------------------------ */
void amq_oracle_gru_step_rb(const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp,
                            const float* alpha_h, int64_t I, int64_t H, int k_w, const float* bias_x,
                            const float* bias_h, const float* x, const float* h_prev, int64_t B,
                            int k_a, int T, const float* g_in, float* g_out, float* h_out) {
  int64_t m = 3 * H;
  double* ax = (double*)malloc(sizeof(double) * (size_t)B * (size_t)m);
  double* ah = (double*)malloc(sizeof(double) * (size_t)B * (size_t)m);
  double* ag = (double*)malloc(sizeof(double) * (size_t)B * (size_t)m);
  float* g = (float*)malloc(sizeof(float) * (size_t)B * (size_t)H);
  preact(Wxp, alpha_x, m, I, k_w, x, B, k_a, T, bias_x, ax);
  preact(Whp, alpha_h, m, H, k_w, h_prev, B, k_a, T, bias_h, ah);
  for (int64_t b = 0; b < B; ++b)
    for (int64_t u = 0; u < H; ++u) {
      double r = sigmoid(ax[b * m + u] + ah[b * m + u]);
      g[b * H + u] = g_in ? g_in[b * H + u] : (float)(r * (double)h_prev[b * H + u]);
      if (g_out) g_out[b * H + u] = g[b * H + u];
    }
  preact(Whp, alpha_h, m, H, k_w, g, B, k_a, T, bias_h, ag);
  for (int64_t b = 0; b < B; ++b)
    for (int64_t u = 0; u < H; ++u) {
      double z = sigmoid(ax[b * m + H + u] + ah[b * m + H + u]);
      double nn = tanh(ax[b * m + 2 * H + u] + ag[b * m + 2 * H + u]);
      h_out[b * H + u] = (float)((1.0 - z) * nn + z * (double)h_prev[b * H + u]);
    }
  free(ax);
  free(ah);
  free(ag);
  free(g);
}

/* ------------------------------------------------------------------ *
 * Variant of Alg. 2 with one more coefficient update (Eq. 5) after the last
 * code assignment, so that the returned coefficients are the least-squares
 * optimum for the returned codes (the algorithm as printed stops after the
 * codes).  Row-wise, packed output as amq_oracle_quantize_rows.
 * ------------------------------------------------------------------ */
void amq_oracle_quantize_rows_final_ls(const float* W, int64_t rows, int64_t cols, int64_t ld, int k,
                                       int T, uint32_t* planes, float* alpha) {
  int64_t wpr = amq_oracle_wpr(cols);
#ifdef _OPENMP
#pragma omp parallel for num_threads(amq_oracle_get_threads()) schedule(static)
#endif
  for (int64_t r = 0; r < rows; ++r) {
    uint8_t* code = (uint8_t*)malloc((size_t)k * (size_t)cols);
    float a[ORACLE_MAX_K];
    amq_oracle_quantize(W + r * ld, cols, k, T, code, a, NULL);
    amq_oracle_ls(W + r * ld, cols, k, code, a);
    for (int i = 0; i < k; ++i) {
      amq_oracle_pack(code + (size_t)i * cols, cols, planes + ((size_t)i * rows + r) * wpr);
      alpha[r * k + i] = a[i];
    }
    free(code);
  }
}

/* ------------------------------------------------------------------ *
 * Reconstruction w_hat = sum_i alpha_i b_i of a row-wise quantization, the
 * quantity the network sees in the forward pass of training (Sec. 4,
 * "Training": w_hat is derived from w and fed to f; the gradient with respect
 * to w is taken equal to the gradient with respect to w_hat).  An entry's
 * value is a code-table value: the binary32 left-to-right sum of +-alpha_i.
 * out: rows x cols with leading dimension ld_out.
 * ------------------------------------------------------------------ */
void amq_oracle_dequantize(const uint32_t* planes, const float* alpha, int64_t rows, int64_t cols,
                           int k, float* out, int64_t ld_out) {
  int64_t wpr = amq_oracle_wpr(cols);
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t l = 0; l < cols; ++l) {
      float v = 0.0f;
      for (int i = 0; i < k; ++i) {
        float term = unpack_bit(planes + ((size_t)i * rows + r) * wpr, l) ? alpha[r * k + i] : -alpha[r * k + i];
        v = (i == 0) ? term : v + term;
      }
      out[r * ld_out + l] = v;
    }
}

/* Clipping of the full-precision weights to [lo, hi] (Sec. 4, "Training":
 * outliers are cut to [-1, 1]). */
void amq_oracle_clip(float* w, int64_t n, float lo, float hi) {
  for (int64_t l = 0; l < n; ++l) w[l] = w[l] < lo ? lo : (w[l] > hi ? hi : w[l]);
}

/* ------------------------------------------------------------------ *
 * Refined greedy approximation (Sec. 2, the comparison method built on
 * Eq. 3-5): for j = 1..k, plane j is the sign of the current residual and
 * alpha_j its mean absolute value (Eq. 4); then all of alpha_1..alpha_j are
 * replaced by the least-squares solution for the first j planes (Eq. 5 on
 * B_j = [b_1 .. b_j]); the next residual is w minus the reconstruction with
 * the refined coefficients.  Codes are never revisited.
 * Precision as everywhere: the reconstruction value of an entry is the
 * binary32 left-to-right sum of +-alpha_i (a code-table value), the residual
 * one binary32 subtraction, the reductions and the solve binary64.  A
 * singular Gram matrix skips that refinement.
 * ------------------------------------------------------------------ */
void amq_oracle_refined_greedy(const float* w, int64_t n, int k, uint8_t* code, float* alpha) {
  float* r = (float*)malloc(sizeof(float) * (size_t)n);
  for (int64_t l = 0; l < n; ++l) r[l] = w[l];
  for (int j = 0; j < k; ++j) {
    double s = 0.0;
    for (int64_t l = 0; l < n; ++l) s += fabs((double)r[l]);
    alpha[j] = (float)(s / (double)n);
    for (int64_t l = 0; l < n; ++l) code[(size_t)j * n + l] = sign_code(r[l]);
    amq_oracle_ls(w, n, j + 1, code, alpha); /* the first j + 1 planes are contiguous in `code` */
    for (int64_t l = 0; l < n; ++l) {
      float v = 0.0f;
      for (int i = 0; i <= j; ++i) {
        float term = code[(size_t)i * n + l] ? alpha[i] : -alpha[i];
        v = (i == 0) ? term : v + term;
      }
      r[l] = w[l] - v;
    }
  }
  free(r);
}

/* Row-wise refined greedy on a matrix, packed output as amq_oracle_quantize_rows. */
void amq_oracle_refined_greedy_rows(const float* W, int64_t rows, int64_t cols, int64_t ld, int k,
                                    uint32_t* planes, float* alpha) {
  int64_t wpr = amq_oracle_wpr(cols);
#ifdef _OPENMP
#pragma omp parallel for num_threads(amq_oracle_get_threads()) schedule(static)
#endif
  for (int64_t r = 0; r < rows; ++r) {
    uint8_t* code = (uint8_t*)malloc((size_t)k * (size_t)cols);
    amq_oracle_refined_greedy(W + r * ld, cols, k, code, alpha + r * k);
    for (int i = 0; i < k; ++i)
      amq_oracle_pack(code + (size_t)i * cols, cols, planes + ((size_t)i * rows + r) * wpr);
    free(code);
  }
}

/* ------------------------------------------------------------------ *
 * Ternary quantization as the constrained 2-bit case (Sec. 2): w ~ a t
 * with t in {-1, 0, +1}^n, i.e. alpha_1 = alpha_2 = a / 2 and
 * t = (b_1 + b_2) / 2.
 *   initial codes: the threshold rule cited there -- entries with
 *     |w_l| <= (0.7 / n) ||w||_1 become 0, the others sign(w_l);
 *   coefficient with the codes fixed: the least-squares a = t^T w / t^T t,
 *     which is the mean of |w_l| over the non-zero entries (t_l w_l = |w_l|);
 *   codes with the coefficient fixed: the nearest of {-a, 0, +a}, i.e.
 *     t_l = sign(w_l) if |w_l| > a / 2, else 0.
 * T alternating cycles {coefficient, codes} follow the initial codes, in
 * the order of Alg. 2; with T = 0 the result is the threshold rule with its
 * own least-squares coefficient.  A set of codes with no non-zero entry
 * leaves the coefficient as it is (0 at the start).
 * Precision: sums in binary64, a and the two thresholds rounded to
 * binary32 ((0.7 * l1) / n evaluated in binary64; a / 2 is exact), every
 * comparison |w_l| > threshold in binary32.
 * Output: t as two code planes (+1 -> 1,1; -1 -> 0,0; 0 -> 1,0) and
 * alpha = {a / 2, a / 2}, the format of the 2-bit quantizer.
 * ------------------------------------------------------------------ */
void amq_oracle_ternary(const float* w, int64_t n, int T, uint8_t* code, float* alpha) {
  double l1 = 0.0;
  for (int64_t l = 0; l < n; ++l) l1 += fabs((double)w[l]);
  float thr = (float)((0.7 * l1) / (double)n);
  float a = 0.0f;
  for (int cycle = 0; cycle <= T; ++cycle) {
    /* codes for the current threshold, and the least-squares coefficient of those codes */
    double s = 0.0;
    int64_t kept = 0;
    for (int64_t l = 0; l < n; ++l) {
      int nz = fabsf(w[l]) > thr;
      code[l] = (uint8_t)(nz ? (w[l] > 0.0f) : 1);
      code[(size_t)n + l] = (uint8_t)(nz ? (w[l] > 0.0f) : 0);
      if (nz) { s += fabs((double)w[l]); ++kept; }
    }
    if (cycle == T) break;              /* the last cycle ends with its codes */
    if (kept > 0) a = (float)(s / (double)kept);
    thr = 0.5f * a;
  }
  /* T = 0: the coefficient that belongs to the initial codes */
  if (T == 0) {
    double s = 0.0;
    int64_t kept = 0;
    for (int64_t l = 0; l < n; ++l)
      if (code[l] == code[(size_t)n + l]) { s += fabs((double)w[l]); ++kept; }
    if (kept > 0) a = (float)(s / (double)kept);
  }
  alpha[0] = 0.5f * a;
  alpha[1] = 0.5f * a;
}

/* Row-wise ternary quantization of a matrix, packed output as amq_oracle_quantize_rows (k = 2). */
void amq_oracle_ternary_rows(const float* W, int64_t rows, int64_t cols, int64_t ld, int T,
                             uint32_t* planes, float* alpha) {
  int64_t wpr = amq_oracle_wpr(cols);
#ifdef _OPENMP
#pragma omp parallel for num_threads(amq_oracle_get_threads()) schedule(static)
#endif
  for (int64_t r = 0; r < rows; ++r) {
    uint8_t* code = (uint8_t*)malloc((size_t)2 * (size_t)cols);
    amq_oracle_ternary(W + r * ld, cols, T, code, alpha + r * 2);
    for (int i = 0; i < 2; ++i)
      amq_oracle_pack(code + (size_t)i * cols, cols, planes + ((size_t)i * rows + r) * wpr);
    free(code);
  }
}

/* ------------------------------------------------------------------ *
 * Relative mean squared error of a row-wise quantization (the measure of
 * Tables 1-2): sum over the matrix of (W - sum_i alpha_i B_i)^2 divided by
 * the sum of W^2, in binary64.  row_err / row_norm (nullable) receive the
 * two sums of every row.
 * ------------------------------------------------------------------ */
double amq_oracle_relative_mse(const float* W, int64_t rows, int64_t cols, int64_t ld, int k,
                               const uint32_t* planes, const float* alpha, double* row_err,
                               double* row_norm) {
  int64_t wpr = amq_oracle_wpr(cols);
  double num = 0.0, den = 0.0;
  for (int64_t r = 0; r < rows; ++r) {
    double e = 0.0, q = 0.0;
    for (int64_t l = 0; l < cols; ++l) {
      double rec = 0.0;
      for (int i = 0; i < k; ++i) {
        int bit = unpack_bit(planes + ((size_t)i * rows + r) * wpr, l);
        rec += bit ? (double)alpha[r * k + i] : -(double)alpha[r * k + i];
      }
      double d = (double)W[r * ld + l] - rec;
      e += d * d;
      q += (double)W[r * ld + l] * (double)W[r * ld + l];
    }
    if (row_err) row_err[r] = e;
    if (row_norm) row_norm[r] = q;
    num += e;
    den += q;
  }
  return num / den;
}

/* ------------------------------------------------------------------ *
 * Operation-count model of Sec. 3-4 (used only by a test that pins the
 * printed speed-up figures).
 *   quantizer:  2 T k^2 n binary, 2 (T + 1) k n non-binary
 *   product:    2 k_w k_h m n + 4 k_h^2 n binary, 6 k_h n + 2 k_w k_h m non-binary
 *   gamma = 2 m n / ( binary / 32 + non-binary )
 * ------------------------------------------------------------------ */
double amq_oracle_gamma(double m, double n, double k_w, double k_h) {
  double bin = 2.0 * k_w * k_h * m * n + 4.0 * k_h * k_h * n;
  double nonbin = 6.0 * k_h * n + 2.0 * k_w * k_h * m;
  return 2.0 * m * n / (bin / 32.0 + nonbin);
}
