// Device-side helpers shared by the gfx950 kernels: wavefront (64-lane) reductions,
// workgroup reductions through LDS, and small utilities.  HIP for CDNA4 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace amq {

constexpr int kWave = 64;

// Phase timers of the profiling build (-DAMQ_PHASE_TIMING, a separate library; see build.py): lane 0
// of every wave of workgroup (0, 0) stores the shader clock at mark `id` in buf[(row0 + wave) * 32 + id];
// the quantizer uses rows 0..7 (AMQ_PHASE), the product kernels rows 8..15 (AMQ_PHASE_B), so that the
// two kernels of one step can be timed in the same run.  In the ordinary build the marks expand to nothing.
#ifdef AMQ_PHASE_TIMING
#define AMQ_PHASE_WHEN(cond, buf, row0, id)                                                     \
  do {                                                                                          \
    if ((buf) && (cond) && (threadIdx.x & 63) == 0)                                             \
      (buf)[((row0) + (threadIdx.x >> 6)) * 32 + (id)] = __builtin_readcyclecounter();          \
  } while (0)
#else
#define AMQ_PHASE_WHEN(cond, buf, row0, id) \
  do {                                      \
  } while (0)
#endif
#define AMQ_PHASE_AT(buf, row0, id) AMQ_PHASE_WHEN(blockIdx.x == 0 && blockIdx.y == 0, buf, row0, id)
#define AMQ_PHASE(buf, id) AMQ_PHASE_AT(buf, 0, id)
#define AMQ_PHASE_B(buf, id) AMQ_PHASE_AT(buf, 8, id)

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

template <int CTRL>
__device__ __forceinline__ float dpp_add(float v) {
  const int t = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true);
  return v + __int_as_float(t);
}

// Sum over aligned groups of 2^lg lanes; every lane of a group ends with the group's total.
__device__ __forceinline__ float group_sum(float v, int lg) {
  if (lg >= 1) v = dpp_add<0xB1>(v);   // quad_perm [1,0,3,2]
  if (lg >= 2) v = dpp_add<0x4E>(v);   // quad_perm [2,3,0,1]
  if (lg >= 3) v = dpp_add<0x141>(v);  // row_half_mirror
  if (lg >= 4) v = dpp_add<0x140>(v);  // row_mirror
  if (lg >= 5) v += __shfl_xor(v, 16, 64);
  if (lg >= 6) v += __shfl_xor(v, 32, 64);
  return v;
}

// ---- operands of the fp4 matrix-core kernels (v_mfma_scale_f32_16x16x128_f8f6f4, E2M1 codes) ----
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));

// 16-byte load marked non-temporal: data that is read once and should not displace what the caches hold.
__device__ __forceinline__ uint4 load_streaming(const uint4* p) {
  const v4i v = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(p));
  return make_uint4((uint32_t)v.x, (uint32_t)v.y, (uint32_t)v.z, (uint32_t)v.w);
}
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kTileB = 16;                         // batch entries per tile
constexpr int kSteps = 8;                          // 1024 entries / 128 per matrix instruction
constexpr int kPlaneBytes = kSteps * kTileB * 64;  // one plane of one tile in LDS: [step][batch entry][k-block][16 B]
constexpr unsigned kNib = 0x22222222u;
constexpr int kScaleOne = 0x7f7f7f7f;              // E8M0 exponent 127 = 2^0 in every byte

// {0, 1} codes: bit p of a packed word -> nibble 0b0010 (1.0 in E2M1) or 0; nibble q of dword s is
// bit 4q + s (a fixed permutation of the 32 entries, the same for both operands of a product).
__device__ __forceinline__ uint4 expand4(uint32_t w) {
  return make_uint4((w << 1) & kNib, w & kNib, (w >> 1) & kNib, (w >> 2) & kNib);
}
// {-1, +1} codes in the same entry order: bit 1 -> 0b0010 (+1.0), bit 0 -> 0b1010 (-1.0).  With both
// operands in this form the matrix instruction returns the inner product of the codes itself (no
// popcount correction).  Entries past the end of a vector must be 0.0 in ONE of the operands:
// expand4_signed_valid clears the nibbles whose bit in `valid` is 0.
__device__ __forceinline__ uint4 expand4_signed(uint32_t w) {
  // (~x & 0x88888888) | 0x22222222 is one three-input bit operation on this target; the bits that a
  // left shift brings in land outside the mask
  auto code = [](uint32_t x) { return (~x & 0x88888888u) | kNib; };
  return make_uint4(code(w << 3), code(w << 2), code(w << 1), code(w));
}
__device__ __forceinline__ uint4 expand4_signed_valid(uint32_t w, uint32_t valid) {
  const uint4 e = expand4_signed(w);
  return make_uint4(e.x & ((valid & 0x11111111u) * 15u), e.y & (((valid >> 1) & 0x11111111u) * 15u),
                    e.z & (((valid >> 2) & 0x11111111u) * 15u), e.w & (((valid >> 3) & 0x11111111u) * 15u));
}
// fp4 operands occupy the first four of the eight operand registers; the rest is left undefined so
// that no registers are spent on it.
__device__ __forceinline__ v8i as_operand(uint4 e) {
  const v4i lo = {(int)e.x, (int)e.y, (int)e.z, (int)e.w};
  return __builtin_shufflevector(lo, lo, 0, 1, 2, 3, -1, -1, -1, -1);
}
__device__ __forceinline__ uint32_t word_of(const uint4 (&q)[2], int t) {
  const uint4 v = q[t >> 2];
  return (t & 3) == 0 ? v.x : (t & 3) == 1 ? v.y : (t & 3) == 2 ? v.z : v.w;
}
// Byte offset, inside one plane of a tile, of the 16 bytes that packed word w of batch entry nn expands
// to: words 4q .. 4q+3 of a row go to k-block q >> 1, steps 4 * (q & 1) + 0..3.
__device__ __forceinline__ int tile_offset_of_word(int w, int nn) {
  const int q = w >> 2;
  return ((4 * (q & 1) + (w & 3)) * kTileB + nn) * 64 + (q >> 1) * 16;
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
