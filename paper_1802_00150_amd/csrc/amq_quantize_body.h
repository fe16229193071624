// Body of the quantizer kernel for one workgroup (Alg. 2 on one vector held in registers, or the copy
// of one row of a quantized table), shared by the stand-alone quantizer kernel and the front kernel of
// the split recurrent step.
#pragma once
#include "amq_launch.h"
#include "amq_quantize_core.h"

namespace amq {

// One workgroup copies row ids[g] of a quantized table (all K planes and coefficients) to
// position g of the output operand; an index outside the table gives the zero vector.
template <int K>
__device__ __forceinline__ void gather_row(const GatherSeg& t, int g, int nthreads) {
  const int wpr = 4 * ((t.n + 127) >> 7);
  const long long id = t.ids[g];
  const bool ok = id >= 0 && id < t.vocab;
  const long long row = ok ? id : 0;
#pragma unroll
  for (int i = 0; i < K; ++i) {
    const uint32_t* src = t.table + ((long long)i * t.vocab + row) * wpr;
    uint32_t* dst = t.planes + ((long long)i * t.count + g) * wpr;
    for (int w = threadIdx.x; w < wpr; w += nthreads) dst[w] = ok ? src[w] : 0u;
  }
  if (threadIdx.x < K) t.coef[(long long)g * K + threadIdx.x] = ok ? t.table_coef[row * K + threadIdx.x] : 0.0f;
}

// vec: index of this workgroup's vector over both segments (then over the gathered rows).  sh: two
// buffers of 16 * kMaxRed doubles of LDS.  Every wave of the workgroup (NW of them) must call this.
template <int K, int NJ, int NW>
__device__ __forceinline__ void quantize_block(const QuantArgs& a, int vec, double (*sh)[16 * kMaxRed]) {
  int phase = 0;
  const int lane = lane_id(), wv = wave_id();
  AMQ_PHASE(AMQ_PHASE_OF(a), 0);
  if (vec >= a.seg[0].count + a.seg[1].count) {
    // workgroups past the vectors to quantize copy table rows by index
    gather_row<K>(a.gather, vec - a.seg[0].count - a.seg[1].count, 64 * NW);
    return;
  }
  const int which = (vec >= a.seg[0].count) ? 1 : 0;
  if (which) vec -= a.seg[0].count;
  const float* X = which ? a.seg[1].X : a.seg[0].X;
  const long long ld = which ? a.seg[1].ld : a.seg[0].ld;
  const int n = which ? a.seg[1].n : a.seg[0].n;
  const int count = which ? a.seg[1].count : a.seg[0].count;
  uint32_t* planes = which ? a.seg[1].planes : a.seg[0].planes;
  float* coef = which ? a.seg[1].coef : a.seg[0].coef;

  const int wpr = 4 * ((n + 127) >> 7);
  const int nslots = wpr >> 1;            // 64-entry slots per row, padding included
  const int nj = (nslots + NW - 1) / NW;  // slots per wave; host guarantees nj <= NJ
  const int base = wv * nj;
  const float* x = X + (long long)vec * ld;

  float w[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int e = (base + j) * 64 + lane;
    w[j] = (j < nj && e < n) ? x[e] : 0.0f;
  }

  float alpha[K];
  unsigned long long mym[K];
  double q[K];
#pragma unroll
  for (int i = 0; i < K; ++i) { alpha[i] = 0.0f; mym[i] = 0ull; q[i] = 0.0; }

  if (a.mode == kQuantLsOnly) {
    // codes given: read the masks, rebuild B^T w from them
#pragma unroll
    for (int i = 0; i < K; ++i) {
      if (lane < nj && base + lane < nslots)
        mym[i] = reinterpret_cast<const unsigned long long*>(planes + ((long long)i * count + vec) * wpr)[base + lane];
      alpha[i] = coef[(long long)vec * K + i];
    }
#pragma unroll
    for (int i = 0; i < K; ++i) {
      double qi = 0.0;
      const int lo = (int)(mym[i] & 0xffffffffull), hi = (int)(mym[i] >> 32);
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        if (j < nj) {
          const unsigned long long mk = ((unsigned long long)(unsigned)__builtin_amdgcn_readlane(hi, j) << 32) |
                                        (unsigned)__builtin_amdgcn_readlane(lo, j);
          const bool bit = (mk >> lane) & 1ull;
          qi += bit ? (double)w[j] : -(double)w[j];
        }
      }
      q[i] = qi;
    }
  } else if (a.mode == kQuantBstOnly) {
#pragma unroll
    for (int i = 0; i < K; ++i) alpha[i] = coef[(long long)vec * K + i];
  }

  AMQ_PHASE(AMQ_PHASE_OF(a), 1);
  quantize_core<K, NJ, NW>(w, n, base, nj, a.mode == kQuantFull, a.mode == kQuantFull ? a.T : 1,
                           a.mode != kQuantBstOnly, a.mode != kQuantLsOnly, alpha, mym, q, sh, phase,
                           AMQ_PHASE_OF(a));

  if (a.mode != kQuantLsOnly) {
#pragma unroll
    for (int i = 0; i < K; ++i)
      if (lane < nj && base + lane < nslots)
        reinterpret_cast<unsigned long long*>(planes + ((long long)i * count + vec) * wpr)[base + lane] = mym[i];
  }
  if (a.mode != kQuantBstOnly && threadIdx.x == 0) {
#pragma unroll
    for (int i = 0; i < K; ++i) coef[(long long)vec * K + i] = alpha[i];
  }
  AMQ_PHASE(AMQ_PHASE_OF(a), 31);
}

}  // namespace amq
