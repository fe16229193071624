// Binary matrix products on packed {-1,+1} codes (Sec. 4, Fig. 3; App. A): xor + popcount
// inner products of every weight plane with every activation plane, then the coefficient
// epilogue.  gfx950, 64-wide wavefronts.
//
// General kernel: a row of one weight plane is wpr/4 16-byte chunks.  The lanes of a wave are
// split into groups of G = pow2ceil(chunks per row) (at most 64); a group owns one row, a lane
// one chunk (looping when a row has more than 64 chunks), so that one wave-wide dwordx4 load
// covers 64/G consecutive rows = up to 1 KiB of contiguous plane memory.  Partial popcounts are
// summed across the group with xor-butterflies; the group's first lane applies
//   y = bias + sum_i alpha_i * sum_j beta_j * (n - 2 * popcount_ij).
#include "amq_device.h"
#include "amq_launch.h"

namespace amq {

namespace {

template <int KW, int KA, int BT>
__global__ __launch_bounds__(256) void bgemm_kernel(GemmArgs a, int lg) {
  const int lane = lane_id(), wv = wave_id();
  const int n = a.op.n;
  const int wpr = 4 * ((n + 127) >> 7);
  const int cpr = wpr >> 2;
  const int G = 1 << lg;
  const int rpw = 64 >> lg;
  const int sub = lane & (G - 1);
  const long long m = a.m;
  const long long row = ((long long)blockIdx.x * 4 + wv) * rpw + (lane >> lg);
  const bool row_ok = row < m;
  const long long rowc = row_ok ? row : m - 1;
  const long long g = blockIdx.y;

  const uint32_t* Wp = a.op.Wp + g * a.g_Wp;
  const float* alpha = a.op.alpha + g * a.g_alpha;
  const uint32_t* Xp = a.op.Xp + g * a.g_Xp;
  const float* beta = a.op.beta + g * a.g_beta;
  const int batch = a.batch;

  for (int b0 = 0; b0 < batch; b0 += BT) {
    int acc[BT][KW][KA];
#pragma unroll
    for (int b = 0; b < BT; ++b)
#pragma unroll
      for (int i = 0; i < KW; ++i)
#pragma unroll
        for (int j = 0; j < KA; ++j) acc[b][i][j] = 0;

    for (int c = sub; c < cpr; c += G) {
      uint4 wq[KW];
#pragma unroll
      for (int i = 0; i < KW; ++i)
        wq[i] = reinterpret_cast<const uint4*>(Wp + ((long long)i * m + rowc) * wpr)[c];
#pragma unroll
      for (int b = 0; b < BT; ++b) {
        const int bb = (b0 + b < batch) ? b0 + b : batch - 1;
#pragma unroll
        for (int j = 0; j < KA; ++j) {
          const uint4 xq = reinterpret_cast<const uint4*>(Xp + ((long long)j * batch + bb) * wpr)[c];
#pragma unroll
          for (int i = 0; i < KW; ++i) acc[b][i][j] += popc4(wq[i], xq);
        }
      }
    }

    for (int o = 1; o < G; o <<= 1) {
#pragma unroll
      for (int b = 0; b < BT; ++b)
#pragma unroll
        for (int i = 0; i < KW; ++i)
#pragma unroll
          for (int j = 0; j < KA; ++j) acc[b][i][j] += __shfl_xor(acc[b][i][j], o, kWave);
    }

    if (sub == 0 && row_ok) {
      float al[KW];
      if (a.Y) {
#pragma unroll
        for (int i = 0; i < KW; ++i) al[i] = alpha[row * KW + i];
      }
      const float bs = (a.Y && a.bias) ? a.bias[row] : 0.0f;
#pragma unroll
      for (int b = 0; b < BT; ++b) {
        if (b0 + b < batch) {
          const long long bb = b0 + b;
          if (a.D) {
#pragma unroll
            for (int i = 0; i < KW; ++i)
#pragma unroll
              for (int j = 0; j < KA; ++j)
                a.D[((bb * m + row) * KW + i) * KA + j] = n - 2 * acc[b][i][j];
          }
          if (a.Y) {
            float* yp = a.Y + g * a.g_Y + bb * m + row;
            float y = a.accumulate ? *yp : 0.0f;
            y += bs;
#pragma unroll
            for (int i = 0; i < KW; ++i) {
              float inner = 0.0f;
#pragma unroll
              for (int j = 0; j < KA; ++j)
                inner = fmaf(beta[bb * KA + j], (float)(n - 2 * acc[b][i][j]), inner);
              y = fmaf(al[i], inner, y);
            }
            *yp = y;
          }
        }
      }
    }
  }
}

template <int KW, int KA>
hipError_t launch_kk(const GemmArgs& a, hipStream_t s) {
  const int wpr = 4 * ((a.op.n + 127) / 128);
  const int cpr = wpr / 4;
  int lg = 0;
  while ((1 << lg) < cpr && lg < 6) ++lg;
  const int rpw = 64 >> lg;
  const long long blocks = (a.m + 4LL * rpw - 1) / (4LL * rpw);
  dim3 grid((unsigned)blocks, (unsigned)a.groups);
  if (a.batch == 1)
    hipLaunchKernelGGL((bgemm_kernel<KW, KA, 1>), grid, dim3(256), 0, s, a, lg);
  else
    hipLaunchKernelGGL((bgemm_kernel<KW, KA, 4>), grid, dim3(256), 0, s, a, lg);
  return hipGetLastError();
}

template <int KW>
hipError_t launch_kw(const GemmArgs& a, hipStream_t s) {
  switch (a.k_a) {
    case 1: return launch_kk<KW, 1>(a, s);
    case 2: return launch_kk<KW, 2>(a, s);
    case 3: return launch_kk<KW, 3>(a, s);
    case 4: return launch_kk<KW, 4>(a, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_gemm(const GemmArgs& a, hipStream_t s) {
  switch (a.k_w) {
    case 1: return launch_kw<1>(a, s);
    case 2: return launch_kw<2>(a, s);
    case 3: return launch_kw<3>(a, s);
    case 4: return launch_kw<4>(a, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace amq
