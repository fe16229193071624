// Alternating multi-bit quantization (Alg. 2) on gfx950: one wavefront (throughput regime,
// many vectors) or one workgroup of NW = 4 wavefronts (latency regime, few vectors) per
// vector, the vector held in registers, every stage of the algorithm in this one kernel.
//
// Element layout in a wave: "slot" j of a lane holds entry (slot_base + j) * 64 + lane, so a
// wave-wide comparison yields, through the 64-bit ballot, exactly two packed code words of
// the exchange format.  Lane j keeps the ballot of slot j; the Gram matrix of Eq. 5 is then a
// per-lane popcount of xor-ed masks plus one integer reduction, and the final store of a plane
// is one coalesced 8-byte-per-lane write.
//
// Precision: stored quantities are binary32; the reductions (sum |r|, B^T w) are accumulated
// in binary64 and the k x k system is solved in binary64 with exact integer cofactors, then
// rounded once.  The comparison "w >= midpoint" that decides a code is binary32.
#include "amq_launch.h"
#include "amq_quantize_core.h"

namespace amq {

namespace {

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

template <int K, int NJ, int NW>
__global__ __launch_bounds__(64 * NW) void quantize_kernel(QuantArgs a) {
  __shared__ double sh[2][16 * kMaxRed];
  int phase = 0;
  const int lane = lane_id(), wv = wave_id();
  AMQ_PHASE(AMQ_PHASE_OF(a), 0);
  asm volatile("" ::AMQ_ARG(a.seg[0].X), AMQ_ARG(a.seg[0].ld), AMQ_ARG(a.seg[0].n), AMQ_ARG(a.seg[0].count),
               AMQ_ARG(a.seg[0].planes), AMQ_ARG(a.seg[0].coef), AMQ_ARG(a.seg[1].X), AMQ_ARG(a.seg[1].ld),
               AMQ_ARG(a.seg[1].n), AMQ_ARG(a.seg[1].count), AMQ_ARG(a.seg[1].planes), AMQ_ARG(a.seg[1].coef),
               AMQ_ARG(a.T), AMQ_ARG(a.mode), AMQ_ARG(a.gather.count));
  int vec = blockIdx.x;
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

template <int K, int NJ, int NW>
void launch_one(QuantArgs a, int total, hipStream_t s) {
  AMQ_PHASE_ATTACH(a);
  hipLaunchKernelGGL((quantize_kernel<K, NJ, NW>), dim3(total), dim3(64 * NW), 0, s, a);
}

// Waves per vector: one when there are enough vectors to fill the chip (throughput regime),
// four when there are few (latency regime: a quarter of the per-entry work per wave, one wave
// per SIMD so that the wave-uniform parts of the algorithm are not replicated on a SIMD); then
// the smallest register bucket that holds the vector's share.  Vectors above 4096 entries
// always take four waves.
template <int K>
hipError_t launch_k(const QuantArgs& a, int max_n, hipStream_t s) {
  const int nvec = a.seg[0].count + a.seg[1].count;
  const int total = nvec + a.gather.count;  // one workgroup per vector, one per gathered row
  if (total == 0) return hipSuccess;
  const int nslots = nvec ? 2 * ((max_n + 127) / 128) : 1;
  int nw = nvec >= 1024 ? 1 : 4;
  // long rows in the throughput regime: four waves of 16 entries per lane keep about 100 registers
  // and four to five waves per SIMD, against more than 250 registers for one wave of 64 entries per
  // lane (measured on 16384 x 4096: 760 -> 513 us at k = 4; two waves of 32 entries per lane:
  // 206 against 175 us at k = 2, 334 against 297 us at k = 3)
  if (nvec >= 1024 && nslots >= 32) nw = 4;
  if (nw > nslots) nw = 1;
  if (nw == 1 && nslots > 64) nw = 4;
  if (nslots > 256) return hipErrorInvalidValue;
  const int nj = (nslots + nw - 1) / nw;
  if (nw == 1) {
    if (nj <= 4) launch_one<K, 4, 1>(a, total, s);
    else if (nj <= 16) launch_one<K, 16, 1>(a, total, s);
    else launch_one<K, 64, 1>(a, total, s);
  } else {
    if (nj <= 1) launch_one<K, 1, 4>(a, total, s);
    else if (nj <= 4) launch_one<K, 4, 4>(a, total, s);
    else if (nj <= 16) launch_one<K, 16, 4>(a, total, s);
    else launch_one<K, 64, 4>(a, total, s);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_quantize(const QuantArgs& a, int k, hipStream_t s) {
  const int max_n = a.seg[1].count > 0 && a.seg[1].n > a.seg[0].n ? a.seg[1].n : a.seg[0].n;
  switch (k) {
    case 1: return launch_k<1>(a, max_n, s);
    case 2: return launch_k<2>(a, max_n, s);
    case 3: return launch_k<3>(a, max_n, s);
    case 4: return launch_k<4>(a, max_n, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace amq
