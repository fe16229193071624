// Device-side helpers shared by the gfx950 kernels: wavefront (64-lane) reductions,
// workgroup reductions through LDS, and small utilities.  HIP for CDNA4 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace amq {

constexpr int kWave = 64;

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }
__device__ __forceinline__ int wave_id() { return threadIdx.x >> 6; }

// Butterfly sums over the 64 lanes; every lane ends with the total.
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// Sum over a workgroup of NW waves.  `scratch` holds NW elements of T in LDS and may be
// reused right after the call returns (two barriers inside).  NW == 1 needs no LDS.
template <int NW, typename T>
__device__ __forceinline__ T block_sum(T v, T* scratch) {
  v = wave_sum(v);
  if constexpr (NW > 1) {
    __syncthreads();
    if (lane_id() == 0) scratch[wave_id()] = v;
    __syncthreads();
    T t = scratch[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) t += scratch[i];
    v = t;
  }
  return v;
}

__device__ __forceinline__ int popc4(uint4 a, uint4 b) {
  return __popc(a.x ^ b.x) + __popc(a.y ^ b.y) + __popc(a.z ^ b.z) + __popc(a.w ^ b.w);
}

// Cell nonlinearities through the hardware exponential (v_exp_f32, ~1 ulp) and reciprocal.
// Absolute error is a few 1e-7, far inside the 1e-4 bar the cell outputs are held to.
__device__ __forceinline__ float sigmoidf_dev(float a) { return __builtin_amdgcn_rcpf(1.0f + __expf(-a)); }
__device__ __forceinline__ float tanhf_dev(float a) {
  const float e = __expf(-2.0f * fabsf(a));  // in (0, 1]: no overflow for any finite a
  return copysignf((1.0f - e) * __builtin_amdgcn_rcpf(1.0f + e), a);
}

// Running log-sum-exp state: (m, s) stands for s * exp(m).  kLseLow is the neutral maximum
// (finite, so that differences never produce NaN).
constexpr float kLseLow = -3.0e38f;
__device__ __forceinline__ void lse_merge(float& m, float& s, float m2, float s2) {
  const float mn = fmaxf(m, m2);
  s = s * __expf(m - mn) + s2 * __expf(m2 - mn);
  m = mn;
}
// Merge over the 64 lanes; every lane ends with the total.
__device__ __forceinline__ void lse_wave_merge(float& m, float& s) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float m2 = __shfl_xor(m, o, kWave), s2 = __shfl_xor(s, o, kWave);
    lse_merge(m, s, m2, s2);
  }
}

}  // namespace amq
