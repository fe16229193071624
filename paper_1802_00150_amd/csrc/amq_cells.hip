// Pointwise parts of the recurrent cells: gate pre-activations -> new state.
// LSTM: Eq. 6 with gate row blocks i, f, o, g (sigmoid, sigmoid, sigmoid, tanh).
// GRU: textbook cell with the reset gate applied to the hidden-side product of the candidate.
#include "amq_device.h"
#include "amq_launch.h"

namespace amq {

namespace {

__global__ __launch_bounds__(256) void lstm_pointwise_kernel(const float* __restrict__ pre,
                                                             const float* c_prev, float* h_out, float* c_out,
                                                             float* hs_out, long long B, long long H) {
  const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= B * H) return;
  const long long b = t / H, u = t - b * H;
  const float* p = pre + b * 4 * H;
  const float gi = sigmoidf_dev(p[u]);
  const float gf = sigmoidf_dev(p[H + u]);
  const float go = sigmoidf_dev(p[2 * H + u]);
  const float gg = tanhf_dev(p[3 * H + u]);
  const float c = fmaf(gf, c_prev[t], gi * gg);
  const float h = go * tanhf_dev(c);
  c_out[t] = c;
  h_out[t] = h;
  if (hs_out) hs_out[t] = h;
}

__global__ __launch_bounds__(256) void gru_pointwise_kernel(const float* __restrict__ pre_x,
                                                            const float* __restrict__ pre_h, const float* h_prev,
                                                            float* h_out, long long B, long long H) {
  const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= B * H) return;
  const long long b = t / H, u = t - b * H;
  const float* px = pre_x + b * 3 * H;
  const float* ph = pre_h + b * 3 * H;
  const float r = sigmoidf_dev(px[u] + ph[u]);
  const float z = sigmoidf_dev(px[H + u] + ph[H + u]);
  const float nn = tanhf_dev(fmaf(r, ph[2 * H + u], px[2 * H + u]));
  h_out[t] = fmaf(z, h_prev[t] - nn, nn);  // (1 - z) * n + z * h_prev
}

// GRU in the original form (reset gate applied to the previous state before the candidate's
// hidden-side product): first the reset gate and g = r * h_prev, later the rest of the cell.
__global__ __launch_bounds__(256) void gru_rb_reset_kernel(const float* __restrict__ pre_x,
                                                           const float* __restrict__ pre_h, const float* h_prev,
                                                           float* g_out, long long B, long long H) {
  const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= B * H) return;
  const long long b = t / H, u = t - b * H;
  const float r = sigmoidf_dev(pre_x[b * 3 * H + u] + pre_h[b * 3 * H + u]);
  g_out[t] = r * h_prev[t];
}

__global__ __launch_bounds__(256) void gru_rb_final_kernel(const float* __restrict__ pre_x,
                                                           const float* __restrict__ pre_h,
                                                           const float* __restrict__ pre_g, const float* h_prev,
                                                           float* h_out, long long B, long long H) {
  const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= B * H) return;
  const long long b = t / H, u = t - b * H;
  const float z = sigmoidf_dev(pre_x[b * 3 * H + H + u] + pre_h[b * 3 * H + H + u]);
  const float nn = tanhf_dev(pre_x[b * 3 * H + 2 * H + u] + pre_g[b * 3 * H + 2 * H + u]);
  h_out[t] = fmaf(z, h_prev[t] - nn, nn);
}

}  // namespace

hipError_t launch_gru_rb_reset(const float* pre_x, const float* pre_h, const float* h_prev, float* g_out, long long B,
                               long long H, hipStream_t s) {
  const long long total = B * H;
  hipLaunchKernelGGL(gru_rb_reset_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, pre_x, pre_h,
                     h_prev, g_out, B, H);
  return hipGetLastError();
}

hipError_t launch_gru_rb_final(const float* pre_x, const float* pre_h, const float* pre_g, const float* h_prev,
                               float* h_out, long long B, long long H, hipStream_t s) {
  const long long total = B * H;
  hipLaunchKernelGGL(gru_rb_final_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, pre_x, pre_h,
                     pre_g, h_prev, h_out, B, H);
  return hipGetLastError();
}

hipError_t launch_lstm_pointwise(const float* pre, const float* c_prev, float* h_out, float* c_out,
                                 float* hs_out, long long B, long long H, hipStream_t s) {
  const long long total = B * H;
  hipLaunchKernelGGL(lstm_pointwise_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, pre,
                     c_prev, h_out, c_out, hs_out, B, H);
  return hipGetLastError();
}

hipError_t launch_gru_pointwise(const float* pre_x, const float* pre_h, const float* h_prev, float* h_out,
                                long long B, long long H, hipStream_t s) {
  const long long total = B * H;
  hipLaunchKernelGGL(gru_pointwise_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, pre_x,
                     pre_h, h_prev, h_out, B, H);
  return hipGetLastError();
}

// Read-only streaming yardstick: every thread walks the buffer with 16-byte loads at a stride of the
// whole grid (each wave-wide load covers 1 KiB of consecutive memory), folds what it reads with xor
// so that nothing can be dropped, and the workgroup leaves one 64-bit word.
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ buf, long long n16,
                                                          unsigned long long* __restrict__ sink) {
  __shared__ unsigned long long part[4];
  // a workgroup takes whole tiles of kTile 16-byte words (32 KiB contiguous), eight loads per lane in flight
  constexpr int kLoads = 8, kTile = 256 * kLoads;
  uint4 acc = make_uint4(0, 0, 0, 0);
  const long long tiles = n16 / kTile;
  for (long long t = blockIdx.x; t < tiles; t += gridDim.x) {
    const uint4* p = buf + t * kTile + threadIdx.x;
    uint4 v[kLoads];
#pragma unroll
    for (int j = 0; j < kLoads; ++j) v[j] = load_streaming(p + j * 256);
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
      acc.x ^= v[j].x; acc.y ^= v[j].y; acc.z ^= v[j].z; acc.w ^= v[j].w;
    }
  }
  for (long long i = tiles * kTile + (long long)blockIdx.x * 256 + threadIdx.x; i < n16; i += (long long)gridDim.x * 256) {
    const uint4 a = buf[i];
    acc.x ^= a.x; acc.y ^= a.y; acc.z ^= a.z; acc.w ^= a.w;
  }
  unsigned long long v = ((unsigned long long)(acc.x ^ acc.z) << 32) | (acc.y ^ acc.w);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v ^= __shfl_xor(v, o, kWave);
  if (lane_id() == 0) part[wave_id()] = v;
  __syncthreads();
  if (threadIdx.x == 0) sink[blockIdx.x] = part[0] ^ part[1] ^ part[2] ^ part[3];
}

hipError_t launch_stream_read(const void* buf, size_t bytes, unsigned long long* sink, hipStream_t s) {
  hipLaunchKernelGGL(stream_read_kernel, dim3(kStreamReadBlocks), dim3(256), 0, s, static_cast<const uint4*>(buf),
                     (long long)(bytes / 16), sink);
  return hipGetLastError();
}

}  // namespace amq
