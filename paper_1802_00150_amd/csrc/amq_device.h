// Device-side helpers shared by the gfx950 kernels: wavefront (64-lane) reductions,
// workgroup reductions through LDS, and small utilities.  HIP for CDNA4 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace amq {

constexpr int kWave = 64;

// Phase timers of the profiling build (-DAMQ_PHASE_TIMING, a separate library; see build.py): lane 0
// of every wave of workgroup (0, 0) stores the shader clock at mark `id` in buf[wave * 32 + id].  In the
// ordinary build the marks expand to nothing.
#ifdef AMQ_PHASE_TIMING
#define AMQ_PHASE(buf, id)                                                                      \
  do {                                                                                          \
    if ((buf) && blockIdx.x == 0 && blockIdx.y == 0 && (threadIdx.x & 63) == 0)                 \
      (buf)[(threadIdx.x >> 6) * 32 + (id)] = __builtin_readcyclecounter();                     \
  } while (0)
#else
#define AMQ_PHASE(buf, id) \
  do {                     \
  } while (0)
#endif

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }
__device__ __forceinline__ int wave_id() { return threadIdx.x >> 6; }

// Kernel arguments arrive through scalar loads that the compiler otherwise issues one by one, each
// just before its first use and each followed by its own wait -- in a latency-bound kernel a chain of
// memory round trips before the first vector load can be issued.  Naming the arguments in one empty
// asm statement at the top of the kernel makes all those loads issue back to back behind one wait.
#define AMQ_ARG(x) "s"(x)

// Workgroup barrier for exchanges through LDS only.  __syncthreads() also orders global memory at
// workgroup scope, which on this target means waiting until every outstanding global load of the wave
// has returned; kernels that keep loads in flight across a staging step use this instead.  LDS writes
// issued before it are visible to the other waves after it; global memory is not ordered by it.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Sum over aligned groups of 8 lanes (DPP, no LDS traffic); every lane of a group ends with the total.
__device__ __forceinline__ int sum8(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xf, 0xf, true);   // quad_perm [1,0,3,2]
  v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xf, 0xf, true);   // quad_perm [2,3,0,1]
  v += __builtin_amdgcn_update_dpp(0, v, 0x141, 0xf, 0xf, true);  // row_half_mirror
  return v;
}

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
