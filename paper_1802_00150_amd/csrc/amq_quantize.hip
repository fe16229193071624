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
#include "amq_quantize_body.h"

namespace amq {

namespace {

// Register budget: the 2-bit kernel of the throughput regime (16 slots per lane) needs 95 registers, one
// bucket above what six waves per SIMD allow; asked for six, the compiler spills four registers and the
// kernel gains 2-3 % (measured on 16384 x 4096: 145 against 148-150 us; eight waves: 176 us).
template <int K, int NJ, int NW>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu((K == 2 && NJ == 16) ? 6 : 1)))
void quantize_kernel(QuantArgs a) {
  __shared__ double sh[2][16 * kMaxRed];
  asm volatile("" ::AMQ_ARG(a.seg[0].X), AMQ_ARG(a.seg[0].ld), AMQ_ARG(a.seg[0].n), AMQ_ARG(a.seg[0].count),
               AMQ_ARG(a.seg[0].planes), AMQ_ARG(a.seg[0].coef), AMQ_ARG(a.seg[1].X), AMQ_ARG(a.seg[1].ld),
               AMQ_ARG(a.seg[1].n), AMQ_ARG(a.seg[1].count), AMQ_ARG(a.seg[1].planes), AMQ_ARG(a.seg[1].coef),
               AMQ_ARG(a.T), AMQ_ARG(a.mode), AMQ_ARG(a.gather.count));
  quantize_block<K, NJ, NW>(a, blockIdx.x, sh);
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
