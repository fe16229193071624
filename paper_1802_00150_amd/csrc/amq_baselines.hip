// The comparison quantizers of Sec. 2 (refined greedy approximation; ternary quantization as the
// 2-bit case with equal coefficients), the relative mean squared error of Tables 1-2, and the
// training-side helpers of Sec. 4 (reconstruction of the quantized
// weights for the forward pass, clipping of the full-precision weights), on gfx950.  Same vector layout and reductions as the alternating quantizer
// (amq_quantize_core.h): one wavefront or one 4-wave workgroup per vector, the vector in registers.
#include "amq_launch.h"
#include "amq_quantize_core.h"

namespace amq {

namespace {

// Stage I of refined greedy for one vector: plane I = sign of the residual, alpha_I = its mean
// absolute value (Eq. 4); then alpha_0..alpha_I are replaced by the least-squares solution for the
// first I + 1 planes (Eq. 5); then the residual is rebuilt from the refined coefficients (the
// reconstruction value of an entry is the binary32 left-to-right sum of +-alpha, as in the code
// table of the alternating quantizer).  s_abs is the l1 norm of the incoming residual.
template <int K, int NJ, int NW, int I>
__device__ __forceinline__ void refined_stage(const float (&w)[NJ], float (&r)[NJ], int n, int base, int nj,
                                              double s_abs, float (&alpha)[K], unsigned long long (&mym)[K],
                                              int (&G)[K][K], double (&qq)[K], double (*sh)[16 * kMaxRed],
                                              int& phase) {
  const int lane = lane_id();
  alpha[I] = (float)(s_abs / (double)n);
  unsigned long long mine = 0ull;
  double q0 = 0.0, q1 = 0.0;
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    if (j < nj) {
      const bool valid = (base + j) * 64 + lane < n;
      const bool bit = valid && (r[j] >= 0.0f);
      const unsigned long long mk = __ballot(bit);
      if (lane == j) mine = mk;
      const double sw = bit ? (double)w[j] : -(double)w[j];
      if (j & 1) q1 += sw; else q0 += sw;
    }
  }
  mym[I] = mine;
  // B^T w of the new plane and its disagreement counts with the earlier planes: one reduction
  double red[1 + I];
  red[0] = q0 + q1;
#pragma unroll
  for (int a = 0; a < I; ++a) red[1 + a] = (double)__popcll(mym[a] ^ mym[I]);
  block_totals<NW, 1 + I>(red, sh, phase);
  qq[I] = red[0];
  G[I][I] = n;
#pragma unroll
  for (int a = 0; a < I; ++a) {
    const int d = __builtin_amdgcn_readfirstlane((int)red[1 + a]);
    G[a][I] = n - 2 * d;
    G[I][a] = G[a][I];
  }
  {
    int Gs[I + 1][I + 1];
    double qs[I + 1];
    float as[I + 1];
#pragma unroll
    for (int a = 0; a <= I; ++a) {
      qs[a] = qq[a];
      as[a] = alpha[a];
#pragma unroll
      for (int c = 0; c <= I; ++c) Gs[a][c] = G[a][c];
    }
    ls_solve<I + 1>(Gs, qs, as);  // a singular Gram matrix leaves the coefficients as they are
#pragma unroll
    for (int a = 0; a <= I; ++a) alpha[a] = as[a];
  }
  if constexpr (I + 1 < K) {
    int lo[I + 1], hi[I + 1];
#pragma unroll
    for (int a = 0; a <= I; ++a) {
      lo[a] = (int)(mym[a] & 0xffffffffull);
      hi[a] = (int)(mym[a] >> 32);
    }
    double s0 = 0.0, s1 = 0.0;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      if (j < nj) {
        const bool valid = (base + j) * 64 + lane < n;
        float v = 0.0f;
#pragma unroll
        for (int a = 0; a <= I; ++a) {
          const unsigned long long mk = ((unsigned long long)(unsigned)__builtin_amdgcn_readlane(hi[a], j) << 32) |
                                        (unsigned)__builtin_amdgcn_readlane(lo[a], j);
          const float term = ((mk >> lane) & 1ull) ? alpha[a] : -alpha[a];
          v = (a == 0) ? term : v + term;
        }
        const float rn = valid ? w[j] - v : 0.0f;
        r[j] = rn;
        if (j & 1) s1 += (double)fabsf(rn); else s0 += (double)fabsf(rn);
      }
    }
    double s[1] = {s0 + s1};
    block_totals<NW, 1>(s, sh, phase);
    refined_stage<K, NJ, NW, I + 1>(w, r, n, base, nj, s[0], alpha, mym, G, qq, sh, phase);
  }
}

template <int K, int NJ, int NW>
__global__ __launch_bounds__(64 * NW) void refined_kernel(const float* X, long long ld, int n, int count,
                                                          uint32_t* planes, float* coef) {
  __shared__ double sh[2][16 * kMaxRed];
  int phase = 0;
  const int lane = lane_id(), wv = wave_id();
  const int vec = blockIdx.x;
  const int wpr = 4 * ((n + 127) >> 7);
  const int nslots = wpr >> 1;
  const int nj = (nslots + NW - 1) / NW;  // host guarantees nj <= NJ
  const int base = wv * nj;
  const float* x = X + (long long)vec * ld;
  float w[NJ], r[NJ];
  double s0 = 0.0, s1 = 0.0;
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int e = (base + j) * 64 + lane;
    w[j] = (j < nj && e < n) ? x[e] : 0.0f;
    r[j] = w[j];
    if (j & 1) s1 += (double)fabsf(w[j]); else s0 += (double)fabsf(w[j]);
  }
  double s[1] = {s0 + s1};
  block_totals<NW, 1>(s, sh, phase);
  float alpha[K];
  unsigned long long mym[K];
  int G[K][K];
  double qq[K];
#pragma unroll
  for (int i = 0; i < K; ++i) { alpha[i] = 0.0f; mym[i] = 0ull; qq[i] = 0.0; }
  refined_stage<K, NJ, NW, 0>(w, r, n, base, nj, s[0], alpha, mym, G, qq, sh, phase);
#pragma unroll
  for (int i = 0; i < K; ++i)
    if (lane < nj && base + lane < nslots)
      reinterpret_cast<unsigned long long*>(planes + ((long long)i * count + vec) * wpr)[base + lane] = mym[i];
  if (threadIdx.x == 0) {
#pragma unroll
    for (int i = 0; i < K; ++i) coef[(long long)vec * K + i] = alpha[i];
  }
}

template <int K, int NJ, int NW>
void launch_refined_one(const float* X, long long ld, int n, int count, uint32_t* planes, float* coef, hipStream_t s) {
  hipLaunchKernelGGL((refined_kernel<K, NJ, NW>), dim3(count), dim3(64 * NW), 0, s, X, ld, n, count, planes, coef);
}

template <int K>
hipError_t launch_refined_k(const float* X, long long ld, int n, int count, uint32_t* planes, float* coef,
                            hipStream_t s) {
  const int nslots = 2 * ((n + 127) / 128);
  if (nslots > 256) return hipErrorInvalidValue;
  // one wave per vector up to 4096 entries when there are many vectors, four waves otherwise
  int nw = (count >= 1024 && nslots <= 64) ? 1 : 4;
  if (nw > nslots) nw = 1;
  const int nj = (nslots + nw - 1) / nw;
  if (nw == 1) {
    if (nj <= 4) launch_refined_one<K, 4, 1>(X, ld, n, count, planes, coef, s);
    else if (nj <= 16) launch_refined_one<K, 16, 1>(X, ld, n, count, planes, coef, s);
    else launch_refined_one<K, 64, 1>(X, ld, n, count, planes, coef, s);
  } else {
    if (nj <= 4) launch_refined_one<K, 4, 4>(X, ld, n, count, planes, coef, s);
    else if (nj <= 16) launch_refined_one<K, 16, 4>(X, ld, n, count, planes, coef, s);
    else launch_refined_one<K, 64, 4>(X, ld, n, count, planes, coef, s);
  }
  return hipGetLastError();
}

// ---- ternary quantization as the 2-bit case with alpha_1 = alpha_2 (Sec. 2) -------------------
// w ~ a t, t in {-1, 0, +1}: initial codes by the threshold (0.7 / n) ||w||_1, then T cycles of
// { a = mean of |w| over the non-zero entries (the least-squares coefficient of the codes),
//   t = sign(w) where |w| > a / 2, else 0 (the nearest of the three levels) }.
// Sums in binary64, thresholds and a in binary32, comparisons in binary32.  Stored as two planes
// (+1 -> 1,1; -1 -> 0,0; 0 -> 1,0) and alpha = {a / 2, a / 2}.
template <int NJ, int NW>
__global__ __launch_bounds__(64 * NW) void ternary_kernel(const float* X, long long ld, int n, int count, int T,
                                                          uint32_t* planes, float* coef) {
  __shared__ double sh[2][16 * kMaxRed];
  int phase = 0;
  const int lane = lane_id(), wv = wave_id();
  const int vec = blockIdx.x;
  const int wpr = 4 * ((n + 127) >> 7);
  const int nslots = wpr >> 1;
  const int nj = (nslots + NW - 1) / NW;  // host guarantees nj <= NJ
  const int base = wv * nj;
  const float* x = X + (long long)vec * ld;
  float w[NJ];
  double s0 = 0.0, s1 = 0.0;
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int e = (base + j) * 64 + lane;
    w[j] = (j < nj && e < n) ? x[e] : 0.0f;   // entries past the end are 0: never above a threshold
    if (j & 1) s1 += (double)fabsf(w[j]); else s0 += (double)fabsf(w[j]);
  }
  double l1[1] = {s0 + s1};
  block_totals<NW, 1>(l1, sh, phase);
  float thr = (float)((0.7 * l1[0]) / (double)n);
  float a = 0.0f;
  for (int cycle = 0; cycle <= T; ++cycle) {
    // the least-squares coefficient of the codes that `thr` defines (also needed after the last
    // codes when T = 0: then it is the coefficient that belongs to the initial codes)
    if (cycle == T && T > 0) break;
    double q0 = 0.0, q1 = 0.0;
    int kept = 0;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      if (j < nj) {
        const float m = fabsf(w[j]);
        const bool nz = m > thr;
        kept += nz ? 1 : 0;
        if (j & 1) q1 += nz ? (double)m : 0.0; else q0 += nz ? (double)m : 0.0;
      }
    }
    double red[2] = {q0 + q1, (double)kept};   // (counts are exact in binary64)
    block_totals<NW, 2>(red, sh, phase);
    if (red[1] > 0.0) a = (float)(red[0] / red[1]);
    if (cycle == T) break;   // T = 0
    thr = 0.5f * a;
  }
  // final codes: lane j of a wave keeps the ballot of its slot j
  unsigned long long m0 = 0ull, m1 = 0ull;
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    if (j < nj) {
      const bool valid = (base + j) * 64 + lane < n;
      const bool nz = fabsf(w[j]) > thr;
      const bool pos = w[j] > 0.0f;
      const unsigned long long b0 = __ballot(valid && (nz ? pos : true));
      const unsigned long long b1 = __ballot(valid && nz && pos);
      if (lane == j) { m0 = b0; m1 = b1; }
    }
  }
  if (lane < nj && base + lane < nslots) {
    reinterpret_cast<unsigned long long*>(planes + ((long long)0 * count + vec) * wpr)[base + lane] = m0;
    reinterpret_cast<unsigned long long*>(planes + ((long long)1 * count + vec) * wpr)[base + lane] = m1;
  }
  if (threadIdx.x == 0) {
    coef[(long long)vec * 2 + 0] = 0.5f * a;
    coef[(long long)vec * 2 + 1] = 0.5f * a;
  }
}

template <int NJ, int NW>
void launch_ternary_one(const float* X, long long ld, int n, int count, int T, uint32_t* planes, float* coef,
                        hipStream_t s) {
  hipLaunchKernelGGL((ternary_kernel<NJ, NW>), dim3(count), dim3(64 * NW), 0, s, X, ld, n, count, T, planes, coef);
}

// ---- relative mean squared error ------------------------------------------------------------
// One wavefront per row: sum over the row of (w - sum_i +-alpha_i)^2 and of w^2, binary64.
template <int K>
__global__ __launch_bounds__(256) void relmse_rows_kernel(const float* W, long long rows, int cols, long long ld,
                                                          const uint32_t* planes, const float* alpha,
                                                          double* row_err, double* row_norm) {
  const long long row = (long long)blockIdx.x * 4 + wave_id();
  if (row >= rows) return;
  const int lane = lane_id();
  const int wpr = 4 * ((cols + 127) >> 7);
  double al[K];
#pragma unroll
  for (int i = 0; i < K; ++i) al[i] = (double)alpha[row * K + i];
  const float* w = W + row * ld;
  double e = 0.0, q = 0.0;
  for (int l = lane; l < cols; l += 64) {
    double rec = 0.0;
#pragma unroll
    for (int i = 0; i < K; ++i) {
      const uint32_t word = planes[((long long)i * rows + row) * wpr + (l >> 5)];
      rec += ((word >> (l & 31)) & 1u) ? al[i] : -al[i];
    }
    const double x = (double)w[l];
    const double d = x - rec;
    e += d * d;
    q += x * x;
  }
  e = wave_sum(e);
  q = wave_sum(q);
  if (lane == 0) {
    row_err[row] = e;
    row_norm[row] = q;
  }
}

// One workgroup adds the per-row sums in a fixed order: result = {error, norm, error / norm}.
__global__ __launch_bounds__(1024) void relmse_final_kernel(const double* row_err, const double* row_norm,
                                                            long long rows, double* result) {
  __shared__ double sh[2][16];
  double e = 0.0, q = 0.0;
  for (long long r = threadIdx.x; r < rows; r += 1024) {
    e += row_err[r];
    q += row_norm[r];
  }
  e = wave_sum(e);
  q = wave_sum(q);
  if (lane_id() == 0) { sh[0][wave_id()] = e; sh[1][wave_id()] = q; }
  __syncthreads();
  if (threadIdx.x == 0) {
    double te = 0.0, tq = 0.0;
    for (int i = 0; i < 16; ++i) { te += sh[0][i]; tq += sh[1][i]; }
    result[0] = te;
    result[1] = tq;
    result[2] = te / tq;
  }
}

// ---- training-side helpers (Sec. 4, "Training") ------------------------------------------------
// One wavefront per row: out[r][l] = binary32 left-to-right sum of +-alpha[r][i].
template <int K>
__global__ __launch_bounds__(256) void dequantize_kernel(const uint32_t* planes, const float* alpha, long long rows,
                                                         int cols, float* out, long long ld_out) {
  const long long row = (long long)blockIdx.x * 4 + wave_id();
  if (row >= rows) return;
  const int lane = lane_id();
  const int wpr = 4 * ((cols + 127) >> 7);
  float al[K];
#pragma unroll
  for (int i = 0; i < K; ++i) al[i] = alpha[row * K + i];
  for (int l0 = 0; l0 < cols; l0 += 64) {
    const int l = l0 + lane;
    float v = 0.0f;
#pragma unroll
    for (int i = 0; i < K; ++i) {
      // the 64 entries of this round are two words of the plane; every lane reads the one it needs
      const uint32_t word = planes[((long long)i * rows + row) * wpr + (l0 >> 5) + (lane >> 5)];
      const float term = ((word >> (lane & 31)) & 1u) ? al[i] : -al[i];
      v = (i == 0) ? term : v + term;
    }
    if (l < cols) out[row * ld_out + l] = v;
  }
}

__global__ __launch_bounds__(256) void clip_kernel(float* w, long long n, float lo, float hi) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i < n) {
    const float v = w[i];
    w[i] = v < lo ? lo : (v > hi ? hi : v);
  }
}

}  // namespace

hipError_t launch_dequantize(const uint32_t* planes, const float* alpha, long long rows, int cols, int k, float* out,
                             long long ld_out, hipStream_t s) {
  const dim3 grid((unsigned)((rows + 3) / 4));
  switch (k) {
    case 1: hipLaunchKernelGGL(dequantize_kernel<1>, grid, dim3(256), 0, s, planes, alpha, rows, cols, out, ld_out); break;
    case 2: hipLaunchKernelGGL(dequantize_kernel<2>, grid, dim3(256), 0, s, planes, alpha, rows, cols, out, ld_out); break;
    case 3: hipLaunchKernelGGL(dequantize_kernel<3>, grid, dim3(256), 0, s, planes, alpha, rows, cols, out, ld_out); break;
    case 4: hipLaunchKernelGGL(dequantize_kernel<4>, grid, dim3(256), 0, s, planes, alpha, rows, cols, out, ld_out); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_clip(float* w, long long n, float lo, float hi, hipStream_t s) {
  hipLaunchKernelGGL(clip_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, w, n, lo, hi);
  return hipGetLastError();
}

hipError_t launch_refined_greedy(const float* X, long long ld, int n, int count, int k, uint32_t* planes, float* coef,
                                 hipStream_t s) {
  switch (k) {
    case 1: return launch_refined_k<1>(X, ld, n, count, planes, coef, s);
    case 2: return launch_refined_k<2>(X, ld, n, count, planes, coef, s);
    case 3: return launch_refined_k<3>(X, ld, n, count, planes, coef, s);
    case 4: return launch_refined_k<4>(X, ld, n, count, planes, coef, s);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_ternary(const float* X, long long ld, int n, int count, int T, uint32_t* planes, float* coef,
                          hipStream_t s) {
  const int nslots = 2 * ((n + 127) / 128);
  if (nslots > 256) return hipErrorInvalidValue;
  // one wave per vector up to 4096 entries when there are many vectors, four waves otherwise
  int nw = (count >= 1024 && nslots <= 64) ? 1 : 4;
  if (nw > nslots) nw = 1;
  const int nj = (nslots + nw - 1) / nw;
  if (nw == 1) {
    if (nj <= 4) launch_ternary_one<4, 1>(X, ld, n, count, T, planes, coef, s);
    else if (nj <= 16) launch_ternary_one<16, 1>(X, ld, n, count, T, planes, coef, s);
    else launch_ternary_one<64, 1>(X, ld, n, count, T, planes, coef, s);
  } else {
    if (nj <= 4) launch_ternary_one<4, 4>(X, ld, n, count, T, planes, coef, s);
    else if (nj <= 16) launch_ternary_one<16, 4>(X, ld, n, count, T, planes, coef, s);
    else launch_ternary_one<64, 4>(X, ld, n, count, T, planes, coef, s);
  }
  return hipGetLastError();
}

hipError_t launch_relative_mse(const float* W, long long rows, int cols, long long ld, int k, const uint32_t* planes,
                               const float* alpha, double* row_err, double* row_norm, double* result,
                               hipStream_t s) {
  const dim3 grid((unsigned)((rows + 3) / 4));
  switch (k) {
    case 1: hipLaunchKernelGGL(relmse_rows_kernel<1>, grid, dim3(256), 0, s, W, rows, cols, ld, planes, alpha, row_err, row_norm); break;
    case 2: hipLaunchKernelGGL(relmse_rows_kernel<2>, grid, dim3(256), 0, s, W, rows, cols, ld, planes, alpha, row_err, row_norm); break;
    case 3: hipLaunchKernelGGL(relmse_rows_kernel<3>, grid, dim3(256), 0, s, W, rows, cols, ld, planes, alpha, row_err, row_norm); break;
    case 4: hipLaunchKernelGGL(relmse_rows_kernel<4>, grid, dim3(256), 0, s, W, rows, cols, ld, planes, alpha, row_err, row_norm); break;
    default: return hipErrorInvalidValue;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(relmse_final_kernel, dim3(1), dim3(1024), 0, s, row_err, row_norm, rows, result);
  return hipGetLastError();
}

}  // namespace amq
