// Whole batch-1 LSTM sequences in one launch, for models whose packed weights fit one compute
// unit (the hidden-300 language model of the paper's PTB experiments: 230 KB of 2-bit planes).
//
// One workgroup of 8 waves runs all time steps of Eq. 6.  The recurrence leaves no parallelism
// across steps, and at this size a step is a few microseconds of work, so kernel launches and
// cross-CU synchronisation would dominate; instead
//   - the input-side planes W_x and both coefficient tables live in LDS (loaded once),
//   - the hidden-side planes W_h live in registers (loaded once; P row passes per wave),
//   - the inputs x_t do not depend on the recurrence: they are quantized ahead of the loop, a
//     chunk of time steps at a time, one wave per vector, into LDS,
//   - per step, all 8 waves quantize h_{t-1} together (the shared quantizer core with 8 waves per
//     vector: 64 entries per wave, reductions through LDS), then form the gate pre-activations
//     of their hidden units (xor + popcount against the packed codes in LDS, coefficients
//     applied per lane, DPP sum over the lanes of a row), apply the cell and write h_t to LDS
//     for the next step; one more barrier closes the step.
// Lane mapping of the products as in the small-batch kernel: groups of G = 2^lg lanes own a
// row (one 16-byte chunk per lane), a wave owns 64 / G hidden units per pass.
#include "amq_launch.h"
#include "amq_quantize_core.h"

namespace amq {

namespace {

constexpr int kSeqWaves = 8;
constexpr int kSeqNJ = 8;  // vectors of at most 512 entries: 8 slots of 64
constexpr size_t kSeqLdsBudget = 150 * 1024;

template <int CTRL>
__device__ __forceinline__ float dpp_addf(float v) {
  const int t = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true);
  return v + __int_as_float(t);
}

__device__ __forceinline__ float group_sumf(float v, int lg) {
  if (lg >= 1) v = dpp_addf<0xB1>(v);   // quad_perm [1,0,3,2]
  if (lg >= 2) v = dpp_addf<0x4E>(v);   // quad_perm [2,3,0,1]
  return v;                             // lg <= 2 here (vectors of at most 512 entries)
}

// One wave quantizes one vector (Alg. 2) and leaves planes [KA][wpr] and coefficients in LDS.
template <int KA>
__device__ __forceinline__ void quantize_to_lds(const float* src, int n, int T, uint32_t* planes, float* coef) {
  const int lane = lane_id();
  const int wpr = 4 * ((n + 127) >> 7);
  const int nslots = wpr >> 1;
  float w[kSeqNJ];
#pragma unroll
  for (int j = 0; j < kSeqNJ; ++j) {
    const int e = j * 64 + lane;
    w[j] = (j < nslots && e < n) ? src[e] : 0.0f;
  }
  float alpha[KA];
  unsigned long long mym[KA];
  double q[KA];
#pragma unroll
  for (int i = 0; i < KA; ++i) { alpha[i] = 0.0f; mym[i] = 0ull; q[i] = 0.0; }
  int phase = 0;
  quantize_core<KA, kSeqNJ, 1>(w, n, 0, nslots, true, T, true, true, alpha, mym, q, nullptr, phase);
#pragma unroll
  for (int i = 0; i < KA; ++i) {
    if (lane < nslots) reinterpret_cast<unsigned long long*>(planes + i * wpr)[lane] = mym[i];
    if (lane == 0) coef[i] = alpha[i];
  }
}

// All 8 waves quantize one vector of at most 512 entries together (wave w owns entries
// 64 w .. 64 w + 63).  Every wave of the workgroup must call this (barriers inside).
template <int KA>
__device__ __forceinline__ void quantize_coop(const float* src, int n, int T, uint32_t* planes, float* coef,
                                              double (*sh)[16 * kMaxRed], int& phase) {
  const int lane = lane_id(), wv = wave_id();
  const int wpr = 4 * ((n + 127) >> 7);
  const int nslots = wpr >> 1;
  float w[1];
  const int e = wv * 64 + lane;
  w[0] = (wv < nslots && e < n) ? src[e] : 0.0f;
  float alpha[KA];
  unsigned long long mym[KA];
  double q[KA];
#pragma unroll
  for (int i = 0; i < KA; ++i) { alpha[i] = 0.0f; mym[i] = 0ull; q[i] = 0.0; }
  quantize_core<KA, 1, kSeqWaves>(w, n, wv, wv < nslots ? 1 : 0, true, T, true, true, alpha, mym, q, sh, phase);
#pragma unroll
  for (int i = 0; i < KA; ++i) {
    if (lane == 0 && wv < nslots) reinterpret_cast<unsigned long long*>(planes + i * wpr)[wv] = mym[i];
    if (threadIdx.x == 0) coef[i] = alpha[i];
  }
}

template <int KW, int KA, int P>
__global__ __launch_bounds__(64 * kSeqWaves) void lstm_seq1_kernel(Seq1Args a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int I = a.I, H = a.H, H4 = 4 * a.H;
  const int cprI = (I + 127) >> 7, cprH = (H + 127) >> 7;
  const int lg = a.lg, G = 1 << lg, R = 64 >> lg;
  const int sub = lane & (G - 1), rloc = lane >> lg;

  // LDS carving (every block a multiple of 16 bytes); seq1_lds_bytes() mirrors this
  uint4* wx4 = reinterpret_cast<uint4*>(smem);                                  // [KW][4H][cprI]
  float* ax = reinterpret_cast<float*>(wx4 + KW * H4 * cprI);                   // [4H][KW]
  float* ah = ax + ((H4 * KW + 3) & ~3);                                        // [4H][KW]
  double (*sh)[16 * kMaxRed] = reinterpret_cast<double (*)[16 * kMaxRed]>(ah + ((H4 * KW + 3) & ~3));
  uint32_t* hp = reinterpret_cast<uint32_t*>(sh + 2);                           // [KA][4 * cprH]
  float* bh = reinterpret_cast<float*>(hp + KA * 4 * cprH);                     // [4]
  float* hbuf = bh + 4;                                                         // [H]
  uint32_t* xp_all = reinterpret_cast<uint32_t*>(hbuf + ((H + 3) & ~3));        // [xchunk][KA][4 * cprI]
  float* bx_all = reinterpret_cast<float*>(xp_all + a.xchunk * KA * 4 * cprI);  // [xchunk][4]

  // ---- one-time loads
  {
    const uint4* src = reinterpret_cast<const uint4*>(a.Wxp);
    const int total = KW * H4 * cprI;
    for (int t = tid; t < total; t += 64 * kSeqWaves) wx4[t] = src[t];
    for (int t = tid; t < H4 * KW; t += 64 * kSeqWaves) { ax[t] = a.ax[t]; ah[t] = a.ah[t]; }
    for (int t = tid; t < H; t += 64 * kSeqWaves) hbuf[t] = a.h[t];
  }
  int unit[P];
  bool ok[P];
  uint4 whq[P][4][KW];
  float bs[P][4], cst[P], hlast[P];
  const uint4* wh4 = reinterpret_cast<const uint4*>(a.Whp);
#pragma unroll
  for (int p = 0; p < P; ++p) {
    unit[p] = (p * kSeqWaves + wv) * R + rloc;
    ok[p] = unit[p] < H;
    const int u = ok[p] ? unit[p] : 0;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
#pragma unroll
      for (int i = 0; i < KW; ++i)
        whq[p][g][i] = (ok[p] && sub < cprH) ? wh4[(i * H4 + g * H + u) * cprH + sub] : make_uint4(0, 0, 0, 0);
      bs[p][g] = a.bias ? a.bias[g * H + u] : 0.0f;
    }
    cst[p] = a.c[u];
    hlast[p] = a.h[u];
  }
  const int leftI = I - 128 * sub, leftH = H - 128 * sub;
  const float bitsI = (float)(leftI < 0 ? 0 : (leftI > 128 ? 128 : leftI));
  const float bitsH = (float)(leftH < 0 ? 0 : (leftH > 128 ? 128 : leftH));
  int phase = 0;
  __syncthreads();

  for (int t0 = 0; t0 < a.steps; t0 += a.xchunk) {
    // ---- quantize the inputs of this chunk of time steps, one wave per vector
    const int tn = (a.steps - t0 < a.xchunk) ? a.steps - t0 : a.xchunk;
    for (int s = wv; s < tn; s += kSeqWaves)
      quantize_to_lds<KA>(a.xs + (long long)(t0 + s) * I, I, a.T, xp_all + s * KA * 4 * cprI, bx_all + s * 4);
    __syncthreads();

    for (int s = 0; s < tn; ++s) {
      // ---- on-line quantization of h_{t-1}, all waves together (barriers inside)
      quantize_coop<KA>(hbuf, H, a.T, hp, bh, sh, phase);
      __syncthreads();

      // ---- products, coefficient epilogue and cell for this lane's hidden units
      const uint4* xp4 = reinterpret_cast<const uint4*>(xp_all + s * KA * 4 * cprI);
      uint4 xq[KA], hq[KA];
      float bxv[KA], bhv[KA];
#pragma unroll
      for (int j = 0; j < KA; ++j) {
        xq[j] = (sub < cprI) ? xp4[j * cprI + sub] : make_uint4(0, 0, 0, 0);
        hq[j] = (sub < cprH) ? reinterpret_cast<const uint4*>(hp)[j * cprH + sub] : make_uint4(0, 0, 0, 0);
        bxv[j] = bx_all[s * 4 + j];
        bhv[j] = bh[j];
      }
#pragma unroll
      for (int p = 0; p < P; ++p) {
        const int u = ok[p] ? unit[p] : 0;
        float pre[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int row = g * H + u;
          float acc = 0.0f;
#pragma unroll
          for (int i = 0; i < KW; ++i) {
            const uint4 wxq = (sub < cprI) ? wx4[(i * H4 + row) * cprI + sub] : make_uint4(0, 0, 0, 0);
            float inx = 0.0f, inh = 0.0f;
#pragma unroll
            for (int j = 0; j < KA; ++j) {
              inx = fmaf(bxv[j], bitsI - 2.0f * (float)popc4(wxq, xq[j]), inx);
              inh = fmaf(bhv[j], bitsH - 2.0f * (float)popc4(whq[p][g][i], hq[j]), inh);
            }
            acc = fmaf(ax[row * KW + i], inx, acc);
            acc = fmaf(ah[row * KW + i], inh, acc);
          }
          pre[g] = group_sumf(acc, lg) + bs[p][g];
        }
        if (sub == 0 && ok[p]) {
          const float gi = sigmoidf_dev(pre[0]);
          const float gf = sigmoidf_dev(pre[1]);
          const float go = sigmoidf_dev(pre[2]);
          const float gg = tanhf_dev(pre[3]);
          const float c = fmaf(gf, cst[p], gi * gg);
          const float h = go * tanhf_dev(c);
          cst[p] = c;
          hlast[p] = h;
          hbuf[unit[p]] = h;
          if (a.hs) a.hs[(long long)(t0 + s) * H + unit[p]] = h;
        }
      }
      __syncthreads();
    }
  }

#pragma unroll
  for (int p = 0; p < P; ++p)
    if (sub == 0 && ok[p]) {
      a.h[unit[p]] = hlast[p];
      a.c[unit[p]] = cst[p];
    }
}

// LDS bytes without the per-step input codes, and bytes of those per time step.
size_t seq1_fixed_lds(int I, int H, int k_w, int k_a) {
  const int cprI = (I + 127) / 128, cprH = (H + 127) / 128;
  size_t b = (size_t)k_w * 4 * H * cprI * 16;            // W_x planes
  b += 2 * (size_t)((4 * H * k_w + 3) & ~3) * 4;        // coefficient tables
  b += 2 * 16 * kMaxRed * sizeof(double);               // reduction scratch
  b += (size_t)k_a * 4 * cprH * 4 + 16;                 // codes and coefficients of h
  b += (size_t)((H + 3) & ~3) * 4;                      // h
  return b;
}
size_t seq1_step_lds(int I, int k_a) { return (size_t)k_a * 4 * ((I + 127) / 128) * 4 + 16; }

template <int KW, int KA, int P>
hipError_t launch_p(const Seq1Args& a, size_t lds, hipStream_t s) {
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&lstm_seq1_kernel<KW, KA, P>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    configured = true;
  }
  hipLaunchKernelGGL((lstm_seq1_kernel<KW, KA, P>), dim3(1), dim3(64 * kSeqWaves), lds, s, a);
  return hipGetLastError();
}

template <int KW, int KA>
hipError_t launch_kk(const Seq1Args& a, int P, size_t lds, hipStream_t s) {
  if constexpr (KW == 2) {
    switch (P) {
      case 1: return launch_p<KW, KA, 1>(a, lds, s);
      case 2: return launch_p<KW, KA, 2>(a, lds, s);
      case 3: return launch_p<KW, KA, 3>(a, lds, s);
      case 4: return launch_p<KW, KA, 4>(a, lds, s);
    }
  } else {
    switch (P) {
      case 1: return launch_p<KW, KA, 1>(a, lds, s);
      case 2: return launch_p<KW, KA, 2>(a, lds, s);
    }
  }
  return hipErrorInvalidValue;
}

int seq1_passes(int I, int H, int* lg_out) {
  const int cpr = ((I > H ? I : H) + 127) / 128;
  int lg = 0;
  while ((1 << lg) < cpr) ++lg;
  *lg_out = lg;
  const int R = 64 >> lg;
  return (H + kSeqWaves * R - 1) / (kSeqWaves * R);
}

}  // namespace

// Batch 1, 2- or 3-bit codes, vectors of at most 512 entries, hidden-side planes within the
// register budget (P * k_w <= 6) and everything else within the LDS budget.
bool lstm_seq1_supported(long long I, long long H, long long B, int k_w, int k_a) {
  if (B != 1 || I > 512 || H > 512 || I <= 0 || H <= 0) return false;
  if (k_w < 2 || k_w > 3 || k_a < 2 || k_a > 3) return false;
  int lg;
  const int P = seq1_passes((int)I, (int)H, &lg);
  if (P * k_w > 6) return false;
  return seq1_fixed_lds((int)I, (int)H, k_w, k_a) + seq1_step_lds((int)I, k_a) <= kSeqLdsBudget;
}

hipError_t launch_lstm_seq1(Seq1Args a, int k_w, int k_a, hipStream_t s) {
  int lg;
  const int P = seq1_passes(a.I, a.H, &lg);
  a.lg = lg;
  // as many time steps of pre-quantized inputs as fit in the LDS budget (at most 64)
  const size_t fixed = seq1_fixed_lds(a.I, a.H, k_w, k_a), per = seq1_step_lds(a.I, k_a);
  long long chunk = (long long)((kSeqLdsBudget - fixed) / per);
  if (chunk > 64) chunk = 64;
  if (chunk > a.steps) chunk = a.steps;
  a.xchunk = (int)chunk;
  const size_t lds = fixed + (size_t)chunk * per;
  if (k_w == 2 && k_a == 2) return launch_kk<2, 2>(a, P, lds, s);
  if (k_w == 2 && k_a == 3) return launch_kk<2, 3>(a, P, lds, s);
  if (k_w == 3 && k_a == 2) return launch_kk<3, 2>(a, P, lds, s);
  if (k_w == 3 && k_a == 3) return launch_kk<3, 3>(a, P, lds, s);
  return hipErrorInvalidValue;
}

}  // namespace amq
