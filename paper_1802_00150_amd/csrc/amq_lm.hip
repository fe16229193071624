// Logarithm of the softmax that closes Eq. 6 (y_t = softmax(W_s h_t + b_s)), one workgroup of
// 16 wavefronts per row of logits.  The row is read once into registers (NV values per lane,
// lane-interleaved so that every load is a coalesced 256-byte wave access), the maximum and the
// sum of exponentials are reduced across the workgroup, and the shifted row is written back.
// Rows longer than 64 * 1024 values take the re-reading variant (three passes, same arithmetic).
// When the product kernel that wrote the logits has already reduced them to per-wave
// (max, sum of exponentials) pairs, only the finishing kernel below runs: it spreads a row over
// many workgroups, which a single workgroup per row (bound by one CU's load path) cannot.
//
// Precision: binary32 throughout; exp through v_exp_f32, the sum of V <= 2^16 positive terms as
// per-lane partial sums + a tree, log through logf.  Absolute error of a result is a few 1e-6.
#include "amq_device.h"
#include "amq_launch.h"

namespace amq {

namespace {

constexpr int kLsmThreads = 1024;
constexpr int kLsmWaves = kLsmThreads / kWave;

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}
__device__ __forceinline__ float wave_sumf(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// Workgroup-wide maximum / sum through LDS; `sh` holds kLsmWaves floats and is free again on return.
template <bool IS_MAX>
__device__ __forceinline__ float block_reduce(float v, float* sh) {
  v = IS_MAX ? wave_max(v) : wave_sumf(v);
  __syncthreads();
  if (lane_id() == 0) sh[wave_id()] = v;
  __syncthreads();
  float t = sh[0];
#pragma unroll
  for (int i = 1; i < kLsmWaves; ++i) t = IS_MAX ? fmaxf(t, sh[i]) : t + sh[i];
  return t;
}

// NV > 0: the row lives in registers.  NV == 0: re-reading variant for any V.
template <int NV>
__global__ __launch_bounds__(kLsmThreads) void log_softmax_kernel(const float* Y, long long V, float* out) {
  __shared__ float sh[kLsmWaves];
  const float* y = Y + (long long)blockIdx.x * V;
  float* o = out + (long long)blockIdx.x * V;
  const int t = threadIdx.x;
  const float kLow = -3.0e38f;
  if constexpr (NV > 0) {
    float v[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const long long e = (long long)j * kLsmThreads + t;
      v[j] = e < V ? y[e] : kLow;
    }
    float mx = kLow;
#pragma unroll
    for (int j = 0; j < NV; ++j) mx = fmaxf(mx, v[j]);
    mx = block_reduce<true>(mx, sh);
    float s = 0.0f;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const long long e = (long long)j * kLsmThreads + t;
      s += e < V ? __expf(v[j] - mx) : 0.0f;
    }
    s = block_reduce<false>(s, sh);
    const float lse = mx + logf(s);
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const long long e = (long long)j * kLsmThreads + t;
      if (e < V) o[e] = v[j] - lse;
    }
  } else {
    float mx = kLow;
    for (long long e = t; e < V; e += kLsmThreads) mx = fmaxf(mx, y[e]);
    mx = block_reduce<true>(mx, sh);
    float s = 0.0f;
    for (long long e = t; e < V; e += kLsmThreads) s += __expf(y[e] - mx);
    s = block_reduce<false>(s, sh);
    const float lse = mx + logf(s);
    for (long long e = t; e < V; e += kLsmThreads) o[e] = y[e] - lse;
  }
}

// Second half of the fused form: the product kernel has left, per row, `slots` pairs
// (max, sum of exp(y - max)) over disjoint parts of the row.  Every workgroup merges the pairs
// of its row (a few KB, from cache) and shifts its own stretch of kFinChunk outputs.
constexpr int kFinThreads = 256;
constexpr int kFinPer = 16;
constexpr int kFinChunk = kFinThreads * kFinPer;
constexpr int kFinRounds = kLseMaxSlots / (8 * kFinThreads);
static_assert(kFinRounds * 8 * kFinThreads == kLseMaxSlots, "slot rounds must cover the maximum exactly");

__global__ __launch_bounds__(kFinThreads) void log_softmax_finish_kernel(const float* Y, long long V,
                                                                        const float* part, int slots, float* out) {
  __shared__ float shm[kFinThreads / kWave], shs[kFinThreads / kWave];
  const int t = threadIdx.x;
  const long long row = blockIdx.y;
  const float* y = Y + row * V;
  float* o = out + row * V;
  const long long e0 = (long long)blockIdx.x * kFinChunk + t;
  float v[kFinPer];
#pragma unroll
  for (int j = 0; j < kFinPer; ++j) {
    const long long e = e0 + (long long)j * kFinThreads;
    v[j] = e < V ? y[e] : 0.0f;
  }
  const float2* pr = reinterpret_cast<const float2*>(part) + row * slots;
  // every pair of the row is requested before the first is used (slots <= kLseMaxSlots, so at
  // most kFinRounds * 8 per thread; rounds past the end are skipped uniformly)
  float2 q[kFinRounds][8];
#pragma unroll
  for (int r = 0; r < kFinRounds; ++r) {
    if (r * 8 * kFinThreads < slots) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int i = (r * 8 + j) * kFinThreads + t;
        q[r][j] = i < slots ? pr[i] : make_float2(kLseLow, 0.0f);
      }
    }
  }
  float m = kLseLow, s = 0.0f;
#pragma unroll
  for (int r = 0; r < kFinRounds; ++r) {
    if (r * 8 * kFinThreads < slots) {
      float mx = m;
#pragma unroll
      for (int j = 0; j < 8; ++j) mx = fmaxf(mx, q[r][j].x);
      float acc = s * __expf(m - mx);
#pragma unroll
      for (int j = 0; j < 8; ++j) acc = fmaf(q[r][j].y, __expf(q[r][j].x - mx), acc);
      m = mx;
      s = acc;
    }
  }
  lse_wave_merge(m, s);
  if (lane_id() == 0) { shm[wave_id()] = m; shs[wave_id()] = s; }
  __syncthreads();
  m = shm[0]; s = shs[0];
#pragma unroll
  for (int i = 1; i < kFinThreads / kWave; ++i) lse_merge(m, s, shm[i], shs[i]);
  const float lse = m + logf(s);
#pragma unroll
  for (int j = 0; j < kFinPer; ++j) {
    const long long e = e0 + (long long)j * kFinThreads;
    if (e < V) o[e] = v[j] - lse;
  }
}

// Scoring: one wave per row merges the row's (max, sum) pairs and writes value - log-sum-exp.
__global__ __launch_bounds__(256) void score_finish_kernel(const float* value, const long long* index, long long B,
                                                           long long V, const float* part, int slots, float* out) {
  const long long row = (long long)blockIdx.x * 4 + wave_id();
  if (row >= B) return;
  const int lane = lane_id();
  const float2* pr = reinterpret_cast<const float2*>(part) + row * slots;
  float m = kLseLow, s = 0.0f;
  for (int i = lane; i < slots; i += kWave) {
    const float2 p = pr[i];
    lse_merge(m, s, p.x, p.y);
  }
  lse_wave_merge(m, s);
  if (lane == 0) {
    const long long ix = index[row];
    out[row] = (ix >= 0 && ix < V) ? value[row] - (m + logf(s)) : __int_as_float(0x7fc00000);
  }
}

__global__ __launch_bounds__(256) void gather_columns_kernel(const float* logprob, long long B, long long V,
                                                             const long long* index, float* out) {
  const long long row = (long long)blockIdx.x * 256 + threadIdx.x;
  if (row >= B) return;
  const long long ix = index[row];
  out[row] = (ix >= 0 && ix < V) ? logprob[row * V + ix] : __int_as_float(0x7fc00000);
}

template <int NV>
void launch_lsm(const float* Y, long long B, long long V, float* out, hipStream_t s) {
  hipLaunchKernelGGL((log_softmax_kernel<NV>), dim3((unsigned)B), dim3(kLsmThreads), 0, s, Y, V, out);
}

}  // namespace

hipError_t launch_log_softmax(const float* Y, long long B, long long V, float* out, hipStream_t s) {
  const long long nv = (V + kLsmThreads - 1) / kLsmThreads;
  if (nv <= 4) launch_lsm<4>(Y, B, V, out, s);
  else if (nv <= 12) launch_lsm<12>(Y, B, V, out, s);
  else if (nv <= 24) launch_lsm<24>(Y, B, V, out, s);
  else if (nv <= 44) launch_lsm<44>(Y, B, V, out, s);
  else if (nv <= 64) launch_lsm<64>(Y, B, V, out, s);
  else launch_lsm<0>(Y, B, V, out, s);
  return hipGetLastError();
}

hipError_t launch_log_softmax_finish(const float* Y, long long B, long long V, const float* part, int slots,
                                     float* out, hipStream_t s) {
  const long long chunks = (V + kFinChunk - 1) / kFinChunk;
  if (B > 65535 || chunks > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(log_softmax_finish_kernel, dim3((unsigned)chunks, (unsigned)B), dim3(kFinThreads), 0, s, Y, V,
                     part, slots, out);
  return hipGetLastError();
}

hipError_t launch_score_finish(const float* value, const long long* index, long long B, long long V, const float* part,
                               int slots, float* out, hipStream_t s) {
  if (B <= 0 || B > (1LL << 31) || slots <= 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(score_finish_kernel, dim3((unsigned)((B + 3) / 4)), dim3(256), 0, s, value, index, B, V, part,
                     slots, out);
  return hipGetLastError();
}

hipError_t launch_gather_columns(const float* logprob, long long B, long long V, const long long* index, float* out,
                                 hipStream_t s) {
  if (B <= 0 || B > (1LL << 31)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(gather_columns_kernel, dim3((unsigned)((B + 255) / 256)), dim3(256), 0, s, logprob, B, V, index,
                     out);
  return hipGetLastError();
}

}  // namespace amq
