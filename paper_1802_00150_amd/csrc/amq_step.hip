// The recurrent step of a sequence whose inputs are all given (Eq. 6 over a sequence, Sec. 4): W_x x_t
// does not depend on the recurrence, so it is taken off the chain h_{t-1} -> quantize -> products -> cell
// -> h_t.  A step is still two launches on one stream, with no synchronisation inside either:
//   front launch of step t: workgroups that quantize h_{t-1} (the chain), workgroups that quantize
//     x_{t+1}, and workgroups that form the x-side sums W_x x_t from the codes the previous front launch
//     left -- three kinds of independent work in one grid, the latter two in the shadow of the first
//     (the quantizer workgroups leave most of the chip idle);
//   back launch of step t: the h-side sums W_h h_{t-1}, plus the stored x-side sums of step t, then the
//     cell -- half the matrix work of a whole step, one wave per SIMD.
// The first step has no codes of x_0 yet: its front launch quantizes h, x_0 and x_1, and its back launch
// is the whole-step kernel.
// The stored x-side sums are exactly the values that the whole-step kernel hands from its x waves to
// the cell, added in the same order: the results are bit-identical to amq_lstm_step's.
#include <atomic>

#include "amq_launch.h"
#include "amq_pair_body.h"
#include "amq_quantize_body.h"

namespace amq {

namespace {

constexpr int kSplitWaves = 4;  // waves per workgroup in both launches (one per SIMD)
constexpr int kSplitNJ = 4;     // slots per lane of the quantizer role: vectors of at most 1024 entries
// (Measured and not kept: front workgroups of 8 waves that each ask for more than half of a compute unit's
// LDS, so that the quantizer of h_{t-1} shares its SIMDs with no x-side wave: 11.9 against 11.8 us per step.)

struct FrontArgs {
  QuantArgs q;      // seg[0] = h_{t-1}; x_{t+1} as seg[1], or as rows to look up in a quantized table (none at the
                    // end of the sequence); at the first step x_0
  QuantArgs q2;     // first step only: x_1
  BmvArgs x;        // x-side product to form (blk[0] only; Y = where the sums go)
  int nx;           // 0 or 1
  int nq, nq2;      // quantizer workgroups = vectors of q and of q2
  int gx;           // row-block groups of the x-side product
  int rowblocks;
};

template <int KW, int KA, int EPI>
__global__ __launch_bounds__(64 * kSplitWaves) void step_front_kernel(FrontArgs f) {
  __shared__ double sh[2][16 * kMaxRed];
  extern __shared__ __attribute__((aligned(16))) uint4 turn[];
  asm volatile("" ::AMQ_ARG(f.q.seg[0].X), AMQ_ARG(f.q.seg[0].ld), AMQ_ARG(f.q.seg[0].n), AMQ_ARG(f.q.seg[0].count),
               AMQ_ARG(f.q.seg[0].planes), AMQ_ARG(f.q.seg[0].coef), AMQ_ARG(f.q.seg[1].X), AMQ_ARG(f.q.seg[1].ld),
               AMQ_ARG(f.q.seg[1].n), AMQ_ARG(f.q.seg[1].count), AMQ_ARG(f.q.seg[1].planes), AMQ_ARG(f.q.seg[1].coef),
               AMQ_ARG(f.q.T), AMQ_ARG(f.q.mode), AMQ_ARG(f.q.gather.count), AMQ_ARG(f.nq), AMQ_ARG(f.nq2), AMQ_ARG(f.gx),
               AMQ_ARG(f.rowblocks));
  const int wg = blockIdx.x;
  if (wg < f.nq) {
    quantize_block<KA, kSplitNJ, kSplitWaves>(f.q, wg, sh);
    return;
  }
  if (wg < f.nq + f.nq2) {
    quantize_block<KA, kSplitNJ, kSplitWaves>(f.q2, wg - f.nq, sh);
    return;
  }
  const int p = wg - f.nq - f.nq2;
  pair_body<KW, KA, 1, EPI, kSplitWaves, kPairXOnly>(f.x, f.rowblocks, p % f.gx, p / f.gx, turn, nullptr);
}

template <int KW, int KA, int EPI>
__global__ __launch_bounds__(64 * kSplitWaves) void step_back_kernel(BmvArgs a, int rowblocks) {
  extern __shared__ __attribute__((aligned(16))) uint4 turn[];
  asm volatile("" ::AMQ_ARG(a.blk[1].Wp), AMQ_ARG(a.blk[1].alpha), AMQ_ARG(a.blk[1].Xp), AMQ_ARG(a.blk[1].beta),
               AMQ_ARG(a.blk[1].n), AMQ_ARG(a.m), AMQ_ARG(a.H), AMQ_ARG(a.batch), AMQ_ARG(a.bias0), AMQ_ARG(a.bias1),
               AMQ_ARG(a.c_prev), AMQ_ARG(a.h_prev), AMQ_ARG(a.h_out), AMQ_ARG(a.c_out), AMQ_ARG(a.hs_out), AMQ_ARG(a.Y),
               AMQ_ARG(rowblocks));
  pair_body<KW, KA, 1, EPI, kSplitWaves, kPairHOnly>(a, rowblocks, blockIdx.x, blockIdx.y, turn, nullptr);
}

template <int KW, int KA, int EPI>
hipError_t front_one(const FrontArgs& f, int grid, hipStream_t s) {
  if constexpr (KW > 3 || KA > 3) {
    return hipErrorInvalidValue;
  } else {
    constexpr size_t lds = pair_body_lds<KW, KA, 1, kSplitWaves, kPairXOnly>();
    static std::atomic<unsigned long long> configured{0};
    hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(&step_front_kernel<KW, KA, EPI>), (int)lds, configured);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((step_front_kernel<KW, KA, EPI>), dim3(grid), dim3(64 * kSplitWaves), lds, s, f);
    return hipGetLastError();
  }
}

template <int KW, int KA, int EPI>
hipError_t back_one(const BmvArgs& a, int rowblocks, hipStream_t s) {
  if constexpr (KW > 3 || KA > 3) {
    return hipErrorInvalidValue;
  } else {
    constexpr size_t lds = pair_body_lds<KW, KA, 1, kSplitWaves, kPairHOnly>();
    static std::atomic<unsigned long long> configured{0};
    hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(&step_back_kernel<KW, KA, EPI>), (int)lds, configured);
    if (e != hipSuccess) return e;
    const dim3 grid((unsigned)((rowblocks + kSplitWaves - 1) / kSplitWaves), (unsigned)((a.batch + kTileB - 1) / kTileB));
    hipLaunchKernelGGL((step_back_kernel<KW, KA, EPI>), grid, dim3(64 * kSplitWaves), lds, s, a, rowblocks);
    return hipGetLastError();
  }
}

template <int KW, int KA>
hipError_t dispatch_epi(const FrontArgs* f, int grid, const BmvArgs* a, int rowblocks, int epi, hipStream_t s) {
  if (epi == kEpiLstm) return f ? front_one<KW, KA, kEpiLstm>(*f, grid, s) : back_one<KW, KA, kEpiLstm>(*a, rowblocks, s);
  if (epi == kEpiGru) return f ? front_one<KW, KA, kEpiGru>(*f, grid, s) : back_one<KW, KA, kEpiGru>(*a, rowblocks, s);
  return hipErrorInvalidValue;
}

template <int KW>
hipError_t dispatch_ka(const FrontArgs* f, int grid, const BmvArgs* a, int rowblocks, int k_a, int epi, hipStream_t s) {
  switch (k_a) {
    case 1: return dispatch_epi<KW, 1>(f, grid, a, rowblocks, epi, s);
    case 2: return dispatch_epi<KW, 2>(f, grid, a, rowblocks, epi, s);
    case 3: return dispatch_epi<KW, 3>(f, grid, a, rowblocks, epi, s);
  }
  return hipErrorInvalidValue;
}

hipError_t dispatch(const FrontArgs* f, int grid, const BmvArgs* a, int rowblocks, int k_w, int k_a, int epi,
                    hipStream_t s) {
  switch (k_w) {
    case 1: return dispatch_ka<1>(f, grid, a, rowblocks, k_a, epi, s);
    case 2: return dispatch_ka<2>(f, grid, a, rowblocks, k_a, epi, s);
    case 3: return dispatch_ka<3>(f, grid, a, rowblocks, k_a, epi, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace

// Where the paired one-tile kernel would take the whole step (few row-block x tile tasks), with codes of
// at most 3 bits.
bool step_split_supported(const BmvArgs& b, int k_w, int k_a, int epi) {
  return mfma4_pair_supported(b, k_w, k_a, epi) && k_a <= 3;
}

hipError_t launch_step_front(const QuantArgs& q, const QuantArgs* q2, const BmvArgs* x, int k_w, int k_a, int epi,
                             hipStream_t s) {
  if (q.mode != kQuantFull) return hipErrorInvalidValue;
  if (q2 && q2->mode != kQuantFull) return hipErrorInvalidValue;
  if (q.seg[0].n > 1024 || (q.seg[1].count > 0 && q.seg[1].n > 1024)) return hipErrorInvalidValue;
  if (q2 && (q2->seg[0].n > 1024 || (q2->seg[1].count > 0 && q2->seg[1].n > 1024))) return hipErrorInvalidValue;
  FrontArgs f{};
  f.q = q;
  AMQ_PHASE_ATTACH(f.q);
  f.nq = q.seg[0].count + q.seg[1].count + q.gather.count;  // (one workgroup per vector and per row to look up)
  if (q2) {
    f.q2 = *q2;
    f.nq2 = q2->seg[0].count + q2->seg[1].count + q2->gather.count;
  }
  int per_x = 0;
  if (x) {
    f.x = *x;
    f.nx = 1;
    f.rowblocks = (int)((x->H + 3) / 4);
    f.gx = (f.rowblocks + kSplitWaves - 1) / kSplitWaves;
    per_x = f.gx * ((x->batch + kTileB - 1) / kTileB);
  }
  return dispatch(&f, f.nq + f.nq2 + per_x, nullptr, 0, k_w, k_a, epi, s);
}

hipError_t launch_step_back(BmvArgs a, int k_w, int k_a, int epi, hipStream_t s) {
  AMQ_PHASE_ATTACH(a);
  return dispatch(nullptr, 0, &a, (int)((a.H + 3) / 4), k_w, k_a, epi, s);
}

}  // namespace amq
