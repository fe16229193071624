// Batched binary matrix products on the matrix cores (Fig. 3 right: the concatenated form),
// general vector length: the int8 kernel that walks K in chunks of 1024 entries.  (Vectors of
// at most 1024 entries take the faster fp4 kernel in amq_mfma4.hip.)
//
// For a batch of concurrent sequences the k_w x k_a plane products are a dense integer
// contraction: M = rows x k_w planes, N = batch x k_a planes, K = vector length.  This kernel
// runs it on v_mfma_i32_16x16x64_i8 (gfx950) with exact int32 accumulation:
//   - weight codes enter as {0,1} bytes, expanded from the packed words in registers with
//     (w >> s) & 0x01010101 (bits s, s+8, s+16, s+24 -> four bytes: a fixed permutation of K);
//   - activation codes enter as {-1,+1} bytes, expanded once per workgroup into LDS with the
//     same permutation of K;
//   - with a in {0,1}, x in {-1,+1}:  sum_l (2a_l - 1) x_l = 2 * sum_l a_l x_l - sum_l x_l, so the
//     +-1 dot product is 2 * acc - sx, sx = 2 * popcount(activation plane) - n.
// A wave owns 16 tile rows x KW planes x 16 batch entries x KA planes (KW*KA accumulators of 4
// registers); a workgroup is 4 waves = 4 row blocks sharing one 16-entry batch tile.  In the
// cell modes the 16 tile rows are 4 hidden units x 4 gates, so that in the 16x16 C layout
// (lane: column = lane % 16, rows 4 * (lane / 16) + 0..3) a lane holds all gates of one unit
// for one batch entry and the LSTM / GRU cell is applied in registers.
#include "amq_device.h"
#include "amq_launch.h"

namespace amq {

namespace {

constexpr int kChunkWords = 32;   // K chunk = 32 words = 1024 entries = 16 MFMA steps

// Values the final step needs besides the products (biases, previous state, old Y), loaded
// early so that their memory latency overlaps the MFMA phase instead of following it.
struct EpiPre {
  float b0[4];
  float b1[4];
  float prev;
  float yold[4];
};

template <int EPI>
__device__ __forceinline__ EpiPre load_pre(const BmvArgs& a, long long rb, int l4, int b, bool bok) {
  EpiPre p;
#pragma unroll
  for (int r = 0; r < 4; ++r) { p.b0[r] = 0.f; p.b1[r] = 0.f; p.yold[r] = 0.f; }
  p.prev = 0.f;
  if constexpr (EPI == kEpiStore) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const long long crow = rb * 16 + 4 * l4 + r;
      if (crow < a.m) {
        if (a.bias0) p.b0[r] = a.bias0[crow];
        if (a.accumulate && a.Y && bok) p.yold[r] = a.Y[(long long)b * a.m + crow];
      }
    }
  } else {
    const long long u = rb * 4 + l4;
    if (u < a.H) {
      constexpr int NG = (EPI == kEpiGru) ? 3 : 4;
#pragma unroll
      for (int r = 0; r < NG; ++r) {
        if (a.bias0) p.b0[r] = a.bias0[r * a.H + u];
        if (EPI == kEpiGru && a.bias1) p.b1[r] = a.bias1[r * a.H + u];
      }
      if (bok) p.prev = (EPI == kEpiLstm) ? a.c_prev[(long long)b * a.H + u] : a.h_prev[(long long)b * a.H + u];
    }
  }
  return p;
}

// Final step for one (row quad, batch entry) in the C view: ysum[block][r] holds the
// coefficient-weighted products of tile rows 4 * l4 + r.  Store mode writes Y; the cell modes
// (tile rows = 4 hidden units x 4 gates) apply Eq. 6 / the GRU cell in registers.
template <int EPI, int NBLK>
__device__ __forceinline__ void cell_or_store(const BmvArgs& a, long long rb, int l4, int b, const float (&ysum)[NBLK][4],
                                              const EpiPre& p) {
  if constexpr (EPI == kEpiStore) {
    if (!a.Y) return;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const long long crow = rb * 16 + 4 * l4 + r;
      if (crow >= a.m) continue;
      a.Y[(long long)b * a.m + crow] = ysum[0][r] + p.b0[r] + p.yold[r];
    }
  } else {
    const long long u = rb * 4 + l4;
    if (u >= a.H) return;
    const long long t = (long long)b * a.H + u;
    if constexpr (EPI == kEpiLstm) {
      float pre[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) pre[r] = ysum[0][r] + ysum[1][r] + p.b0[r];
      const float gi = sigmoidf_dev(pre[0]);
      const float gf = sigmoidf_dev(pre[1]);
      const float go = sigmoidf_dev(pre[2]);
      const float gg = tanhf_dev(pre[3]);
      const float c = fmaf(gf, p.prev, gi * gg);
      const float h = go * tanhf_dev(c);
      a.c_out[t] = c;
      a.h_out[t] = h;
      if (a.hs_out) a.hs_out[t] = h;
    } else {
      const float rg = sigmoidf_dev(ysum[0][0] + ysum[1][0] + p.b0[0] + p.b1[0]);
      const float z = sigmoidf_dev(ysum[0][1] + ysum[1][1] + p.b0[1] + p.b1[1]);
      const float nn = tanhf_dev(fmaf(rg, ysum[1][2] + p.b1[2], ysum[0][2] + p.b0[2]));
      a.h_out[t] = fmaf(z, p.prev - nn, nn);
    }
  }
}

template <int KW, int KA, int EPI>
__global__ __launch_bounds__(256) void mfma_kernel(BmvArgs a) {
  // activation tile: [plane][step t][batch entry][64 bytes = 4 k-blocks x 16]
  __shared__ __attribute__((aligned(16))) unsigned char btile[KA * 16 * kTileB * 64];
  __shared__ int pops[2][KA][kTileB];
  constexpr int NBLK = (EPI == kEpiStore) ? 1 : 2;
  constexpr int NG = (EPI == kEpiGru) ? 3 : 4;
  constexpr unsigned kByteLsb = 0x01010101u;

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int l16 = lane & 15, l4 = lane >> 4;
  const long long rb = (long long)blockIdx.x * 4 + wv;  // row block of this wave
  const int b0 = blockIdx.y * kTileB;
  const int batch = a.batch;

  // A-operand view: lane = (tile row l16, k-block l4)
  long long wrow;
  bool wok;
  if constexpr (EPI == kEpiStore) {
    wrow = rb * 16 + l16;
    wok = wrow < a.m;
  } else {
    const long long unit = rb * 4 + (l16 >> 2);
    const int gate = l16 & 3;
    wok = unit < a.H && gate < NG;
    wrow = (long long)gate * a.H + unit;
  }
  if (!wok) wrow = 0;
  const int half = l4 >> 1;        // which 16 words of the 32-word chunk
  const int sh0 = 4 * (l4 & 1);    // which 4 of the 8 bit-strides
  const EpiPre pre = load_pre<EPI>(a, rb, l4, b0 + l16, b0 + l16 < batch);

  float ysum[NBLK][4];
#pragma unroll
  for (int k = 0; k < NBLK; ++k)
#pragma unroll
    for (int r = 0; r < 4; ++r) ysum[k][r] = 0.0f;

#pragma unroll
  for (int k = 0; k < NBLK; ++k) {
    const int n = a.blk[k].n;
    const int wpr = 4 * ((n + 127) >> 7);
    const int nkc = (wpr + kChunkWords - 1) / kChunkWords;
    const uint32_t* Wp = a.blk[k].Wp;
    const uint32_t* Xp = a.blk[k].Xp;

    v4i acc[KW][KA];
#pragma unroll
    for (int i = 0; i < KW; ++i)
#pragma unroll
      for (int j = 0; j < KA; ++j) acc[i][j] = v4i{0, 0, 0, 0};
    if (tid < KA * kTileB) pops[k][tid / kTileB][tid % kTileB] = 0;

    for (int kc = 0; kc < nkc; ++kc) {
      // this lane's 16 weight words per plane for the chunk, pre-shifted to its bit-strides
      uint32_t aw[KW][16];
      const int wbase = kc * kChunkWords + 16 * half;
#pragma unroll
      for (int i = 0; i < KW; ++i) {
        const uint32_t* rowp = Wp + ((long long)i * a.m + wrow) * wpr;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          uint4 t4 = make_uint4(0, 0, 0, 0);
          if (wok && wbase + 4 * v < wpr) t4 = reinterpret_cast<const uint4*>(rowp)[(wbase >> 2) + v];
          aw[i][4 * v + 0] = t4.x >> sh0;
          aw[i][4 * v + 1] = t4.y >> sh0;
          aw[i][4 * v + 2] = t4.z >> sh0;
          aw[i][4 * v + 3] = t4.w >> sh0;
        }
      }
      __syncthreads();  // previous tile consumed (and pops zeroed)
      // expand the activation tile of this chunk into LDS as +-1 bytes
      for (int e = tid; e < KA * kTileB * kChunkWords; e += 256) {
        const int nn = e & (kTileB - 1);
        const int wi = (e >> 4) & (kChunkWords - 1);
        const int j = e >> 9;
        const int b = b0 + nn;
        const int gw = kc * kChunkWords + wi;
        const bool valid = b < batch && gw < wpr;
        uint32_t w = 0;
        if (valid) {
          w = Xp[((long long)j * batch + b) * wpr + gw];
          atomicAdd(&pops[k][j][nn], __popc(w));
        }
        uint32_t ev[8];
#pragma unroll
        for (int s = 0; s < 8; ++s) ev[s] = valid ? ~(((w >> s) & kByteLsb) * 0xFEu) : 0u;  // 1 -> 0x01, 0 -> 0xFF
        const int t = wi & 15, p = wi >> 4;
        uint4* dst = reinterpret_cast<uint4*>(btile + (((j * 16 + t) * kTileB + nn) * 64 + p * 32));
        dst[0] = make_uint4(ev[0], ev[1], ev[2], ev[3]);
        dst[1] = make_uint4(ev[4], ev[5], ev[6], ev[7]);
      }
      __syncthreads();
#pragma unroll
      for (int t = 0; t < 16; ++t) {
        v4i bop[KA];
#pragma unroll
        for (int j = 0; j < KA; ++j)
          bop[j] = *reinterpret_cast<const v4i*>(btile + (((j * 16 + t) * kTileB + l16) * 64 + l4 * 16));
#pragma unroll
        for (int i = 0; i < KW; ++i) {
          const uint32_t w = aw[i][t];
          v4i aop;
          aop.x = (int)(w & kByteLsb);
          aop.y = (int)((w >> 1) & kByteLsb);
          aop.z = (int)((w >> 2) & kByteLsb);
          aop.w = (int)((w >> 3) & kByteLsb);
#pragma unroll
          for (int j = 0; j < KA; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(aop, bop[j], acc[i][j], 0, 0, 0);
        }
      }
    }

    // MFMAs read all 64 lanes; keep them (and the code feeding them) out of the divergent
    // branches of the epilogue by pinning the accumulators in uniform control flow.
#pragma unroll
    for (int i = 0; i < KW; ++i)
#pragma unroll
      for (int j = 0; j < KA; ++j) asm volatile("" : "+v"(acc[i][j]));
    // block epilogue in the C view: lane = (batch column l16, row quad l4)
    const int b = b0 + l16;
    const bool bok = b < batch;
    int sx[KA];
    float bt[KA];
#pragma unroll
    for (int j = 0; j < KA; ++j) {
      sx[j] = 2 * pops[k][j][l16] - n;
      bt[j] = (bok && a.blk[k].beta) ? a.blk[k].beta[(long long)b * KA + j] : 0.0f;
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      long long crow;
      bool cok;
      if constexpr (EPI == kEpiStore) {
        crow = rb * 16 + 4 * l4 + r;
        cok = crow < a.m;
      } else {
        const long long unit = rb * 4 + l4;
        cok = unit < a.H && r < NG;
        crow = (long long)r * a.H + unit;
      }
      if (!cok) continue;
      float y = 0.0f;
#pragma unroll
      for (int i = 0; i < KW; ++i) {
        float inner = 0.0f;
#pragma unroll
        for (int j = 0; j < KA; ++j) {
          const int d = 2 * acc[i][j][r] - sx[j];
          if (EPI == kEpiStore && a.D && bok) a.D[(((long long)b * a.m + crow) * KW + i) * KA + j] = d;
          inner = fmaf(bt[j], (float)d, inner);
        }
        if (a.blk[k].alpha) y = fmaf(a.blk[k].alpha[crow * KW + i], inner, y);
      }
      ysum[k][r] = y;
    }
  }

  const int b = b0 + l16;
  if (b >= batch) return;
  cell_or_store<EPI, NBLK>(a, rb, l4, b, ysum, pre);
}

template <int KW, int KA, int EPI>
hipError_t launch_mode(const BmvArgs& a, hipStream_t s) {
  const long long rowblocks = (EPI == kEpiStore) ? (a.m + 15) / 16 : (a.H + 3) / 4;
  const long long btiles = (a.batch + kTileB - 1) / kTileB;
  dim3 grid((unsigned)((rowblocks + 3) / 4), (unsigned)btiles);
  hipLaunchKernelGGL((mfma_kernel<KW, KA, EPI>), grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

template <int KW, int KA>
hipError_t launch_epi(const BmvArgs& a, int epi, hipStream_t s) {
  switch (epi) {
    case kEpiStore: return launch_mode<KW, KA, kEpiStore>(a, s);
    case kEpiLstm: return launch_mode<KW, KA, kEpiLstm>(a, s);
    case kEpiGru: return launch_mode<KW, KA, kEpiGru>(a, s);
  }
  return hipErrorInvalidValue;
}

template <int KW>
hipError_t launch_ka(const BmvArgs& a, int k_a, int epi, hipStream_t s) {
  switch (k_a) {
    case 1: return launch_epi<KW, 1>(a, epi, s);
    case 2: return launch_epi<KW, 2>(a, epi, s);
    case 3: return launch_epi<KW, 3>(a, epi, s);
    case 4: return launch_epi<KW, 4>(a, epi, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace

bool mfma_supported(long long batch) { return batch <= 65535LL * kTileB; }

hipError_t launch_mfma(const BmvArgs& a, int k_w, int k_a, int epi, hipStream_t s) {
  switch (k_w) {
    case 1: return launch_ka<1>(a, k_a, epi, s);
    case 2: return launch_ka<2>(a, k_a, epi, s);
    case 3: return launch_ka<3>(a, k_a, epi, s);
    case 4: return launch_ka<4>(a, k_a, epi, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace amq
