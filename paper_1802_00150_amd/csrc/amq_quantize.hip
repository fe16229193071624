// Alternating multi-bit quantization (Alg. 2) on gfx950: one wavefront (throughput regime,
// many vectors) or one workgroup of NW = 4 / 16 wavefronts (latency regime, few vectors) per
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
#include "amq_device.h"
#include "amq_launch.h"

namespace amq {

namespace {

template <int N>
__device__ __forceinline__ long long idet(const long long* m) {
  if constexpr (N == 1) {
    return m[0];
  } else if constexpr (N == 2) {
    return m[0] * m[3] - m[1] * m[2];
  } else {
    long long d = 0;
#pragma unroll
    for (int c = 0; c < N; ++c) {
      long long sub[(N - 1) * (N - 1)];
#pragma unroll
      for (int i = 1; i < N; ++i) {
        int cc = 0;
#pragma unroll
        for (int j = 0; j < N; ++j) {
          if (j == c) continue;
          sub[(i - 1) * (N - 1) + cc] = m[i * N + j];
          ++cc;
        }
      }
      long long t = m[c] * idet<N - 1>(sub);
      d += (c & 1) ? -t : t;
    }
    return d;
  }
}

// Eq. 5 for one vector: alpha = G^{-1} q with G the integer Gram matrix of the codes.
// G^{-1} = adj(G) / det(G) with exact integer cofactors (|entries| <= n <= 16384, K <= 4 fits
// 64-bit).  A singular G leaves alpha unchanged.
template <int K>
__device__ __forceinline__ void ls_solve(const int (&G)[K][K], const double (&q)[K], float (&alpha)[K]) {
  if constexpr (K == 1) {
    alpha[0] = (float)(q[0] / (double)G[0][0]);
  } else {
    long long m[K * K];
#pragma unroll
    for (int i = 0; i < K; ++i)
#pragma unroll
      for (int j = 0; j < K; ++j) m[i * K + j] = G[i][j];
    // cofactors of the first column give the determinant; all cofactors give the adjugate
    long long cof[K][K];
#pragma unroll
    for (int i = 0; i < K; ++i)
#pragma unroll
      for (int j = 0; j < K; ++j) {
        long long sub[(K - 1) * (K - 1)];
        int rr = 0;
#pragma unroll
        for (int a = 0; a < K; ++a) {
          if (a == i) continue;
          int cc = 0;
#pragma unroll
          for (int b = 0; b < K; ++b) {
            if (b == j) continue;
            sub[rr * (K - 1) + cc] = m[a * K + b];
            ++cc;
          }
          ++rr;
        }
        long long d = idet<K - 1>(sub);
        cof[i][j] = ((i + j) & 1) ? -d : d;
      }
    long long det = 0;
#pragma unroll
    for (int j = 0; j < K; ++j) det += m[j] * cof[0][j];
    if (det == 0) return;
    const double inv = 1.0 / (double)det;
#pragma unroll
    for (int i = 0; i < K; ++i) {
      // adj = cof^T; G symmetric so cof is symmetric too, but keep the general form
      double s = 0.0;
#pragma unroll
      for (int j = 0; j < K; ++j) s += (double)cof[j][i] * q[j];
      alpha[i] = (float)(s * inv);
    }
  }
}

__device__ __forceinline__ float readlane_f(float v, int l) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l));
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_d(double v) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = __builtin_amdgcn_update_dpp(0, lo, CTRL, ROW_MASK, 0xf, false);
  hi = __builtin_amdgcn_update_dpp(0, hi, CTRL, ROW_MASK, 0xf, false);
  return __hiloint2double(hi, lo);
}

// Totals of NV doubles over the 64 lanes through DPP (no LDS traffic); the results are
// wave-uniform (read from lane 63).  The NV chains are independent and interleave.
template <int NV>
__device__ __forceinline__ void wave_totals(double (&v)[NV]) {
#pragma unroll
  for (int i = 0; i < NV; ++i) v[i] += dpp_d<0xB1, 0xf>(v[i]);   // quad_perm [1,0,3,2]
#pragma unroll
  for (int i = 0; i < NV; ++i) v[i] += dpp_d<0x4E, 0xf>(v[i]);   // quad_perm [2,3,0,1]
#pragma unroll
  for (int i = 0; i < NV; ++i) v[i] += dpp_d<0x141, 0xf>(v[i]);  // row_half_mirror
#pragma unroll
  for (int i = 0; i < NV; ++i) v[i] += dpp_d<0x140, 0xf>(v[i]);  // row_mirror: every lane holds its row's sum
#pragma unroll
  for (int i = 0; i < NV; ++i) v[i] += dpp_d<0x142, 0xa>(v[i]);  // row_bcast15 into rows 1 and 3
#pragma unroll
  for (int i = 0; i < NV; ++i) v[i] += dpp_d<0x143, 0xc>(v[i]);  // row_bcast31 into rows 2 and 3
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int lo = __builtin_amdgcn_readlane(__double2loint(v[i]), 63);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v[i]), 63);
    v[i] = __hiloint2double(hi, lo);
  }
}

constexpr int kMaxRed = 10;  // K coefficients + K(K-1)/2 plane pairs at K = 4

// Totals over the whole workgroup; one barrier per call, two LDS buffers used alternately.
template <int NW, int NV>
__device__ __forceinline__ void block_totals(double (&v)[NV], double (*sh)[16 * kMaxRed], int& phase) {
  wave_totals<NV>(v);
  if constexpr (NW > 1) {
    const int wv = wave_id();
    if (lane_id() == 0) {
#pragma unroll
      for (int i = 0; i < NV; ++i) sh[phase][wv * NV + i] = v[i];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      double t = sh[phase][i];
#pragma unroll
      for (int w = 1; w < NW; ++w) t += sh[phase][w * NV + i];
      v[i] = t;
    }
    phase ^= 1;
  }
}

template <int K, int NJ, int NW>
__global__ __launch_bounds__(64 * NW) void quantize_kernel(QuantArgs a) {
  __shared__ double sh[2][16 * kMaxRed];
  int phase = 0;
  constexpr int M = 1 << K;
  constexpr int NP = K * (K - 1) / 2;
  const int lane = lane_id(), wv = wave_id();
  int vec = blockIdx.x;
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
  const double dn = (double)n;

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

  if (a.mode == kQuantFull) {
    // ---- greedy initialisation, Eq. 4.  One pass per stage: it assigns the signs, updates the
    // residual and accumulates the l1 norm of the new residual for the next stage.
    float r[NJ];
    double s[1];
    {
      double s0 = 0.0, s1 = 0.0;
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        r[j] = w[j];
        if (j & 1) s1 += (double)fabsf(w[j]); else s0 += (double)fabsf(w[j]);
      }
      s[0] = s0 + s1;
    }
    block_totals<NW, 1>(s, sh, phase);
#pragma unroll
    for (int i = 0; i < K; ++i) {
      const float al = (float)(s[0] / dn);
      alpha[i] = al;
      unsigned long long mine = 0ull;
      double q0 = 0.0, q1 = 0.0, s0 = 0.0, s1 = 0.0;
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        if (j < nj) {
          const bool valid = (base + j) * 64 + lane < n;
          const bool bit = valid && (r[j] >= 0.0f);
          const unsigned long long mk = __ballot(bit);
          if (lane == j) mine = mk;
          const double sw = bit ? (double)w[j] : -(double)w[j];
          const float rn = valid ? r[j] - (bit ? al : -al) : 0.0f;
          r[j] = rn;
          if (j & 1) { q1 += sw; s1 += (double)fabsf(rn); } else { q0 += sw; s0 += (double)fabsf(rn); }
        }
      }
      mym[i] = mine;
      q[i] = q0 + q1;
      if (i + 1 < K) {
        s[0] = s0 + s1;
        block_totals<NW, 1>(s, sh, phase);
      }
    }
  } else if (a.mode == kQuantLsOnly) {
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
  } else {
#pragma unroll
    for (int i = 0; i < K; ++i) alpha[i] = coef[(long long)vec * K + i];
  }

  const int iters = (a.mode == kQuantFull) ? a.T : 1;
  for (int it = 0; it < iters; ++it) {
    if (a.mode != kQuantBstOnly) {
      // ---- coefficients with the codes fixed, Eq. 5: B^T w and the disagreement counts of
      // every plane pair go through one workgroup reduction (counts are exact in binary64)
      double red[K + NP];
#pragma unroll
      for (int i = 0; i < K; ++i) red[i] = q[i];
      {
        int t = K;
#pragma unroll
        for (int i = 0; i < K; ++i)
#pragma unroll
          for (int j = i + 1; j < K; ++j) red[t++] = (double)__popcll(mym[i] ^ mym[j]);
      }
      block_totals<NW, K + NP>(red, sh, phase);
      int G[K][K];
      double qq[K];
      {
        int t = K;
#pragma unroll
        for (int i = 0; i < K; ++i) {
          qq[i] = red[i];
          G[i][i] = n;
#pragma unroll
          for (int j = i + 1; j < K; ++j) {
            const int d = __builtin_amdgcn_readfirstlane((int)red[t++]);  // wave-uniform: integer math on the scalar unit
            G[i][j] = n - 2 * d;
            G[j][i] = G[i][j];
          }
        }
      }
      ls_solve<K>(G, qq, alpha);
      if (a.mode == kQuantLsOnly) break;
    }

    // ---- code table in ascending order (Alg. 2) built across lanes: lane p < 2^K owns the
    // pattern p (coefficient i positive iff bit K-1-i of p), ranks itself among all values
    // (ties by pattern), and pushes (value, pattern) to the lane of its rank.
    const int p = lane & (M - 1);
    float v = 0.0f;
#pragma unroll
    for (int i = 0; i < K; ++i) {
      const float term = ((p >> (K - 1 - i)) & 1) ? alpha[i] : -alpha[i];
      v = (i == 0) ? term : v + term;
    }
    int rank = 0;
#pragma unroll
    for (int o = 0; o < M; ++o) {
      const float vo = readlane_f(v, o);
      rank += (vo < v || (vo == v && o < p)) ? 1 : 0;
    }
    if (lane >= M) rank = lane;
    const float sv = __int_as_float(__builtin_amdgcn_ds_permute(rank << 2, __float_as_int(v)));
    const int sp = __builtin_amdgcn_ds_permute(rank << 2, p);
    float thr[M - 1];  // midpoints of adjacent codes, wave-uniform
#pragma unroll
    for (int j = 0; j < M - 1; ++j) thr[j] = 0.5f * (readlane_f(sv, j) + readlane_f(sv, j + 1));
    unsigned bm[K];  // bit `pos` of bm[i]: plane i is +1 for the code at sorted position pos
#pragma unroll
    for (int i = 0; i < K; ++i) bm[i] = (unsigned)__ballot(lane < M && ((sp >> (K - 1 - i)) & 1));

    // ---- codes with the coefficients fixed (Alg. 1); the position in the sorted table is the
    // number of midpoints <= w, which is where the k-comparison tree walk ends.
    const bool more = (a.mode == kQuantFull) && (it + 1 < iters);  // B^T w is needed by another cycle
    unsigned long long mine[K];
    double qa[K], qb[K];
#pragma unroll
    for (int i = 0; i < K; ++i) { mine[i] = 0ull; qa[i] = 0.0; qb[i] = 0.0; }
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      if (j < nj) {
        const bool valid = (base + j) * 64 + lane < n;
        int pos = 0;
#pragma unroll
        for (int t = 0; t < M - 1; ++t) pos += (w[j] >= thr[t]) ? 1 : 0;
        const double wd = (double)w[j];
#pragma unroll
        for (int i = 0; i < K; ++i) {
          const bool bit = valid && ((bm[i] >> pos) & 1u);
          const unsigned long long mk = __ballot(bit);
          if (lane == j) mine[i] = mk;
          if (more) {
            if (j & 1) qb[i] += bit ? wd : -wd; else qa[i] += bit ? wd : -wd;
          }
        }
      }
    }
#pragma unroll
    for (int i = 0; i < K; ++i) { mym[i] = mine[i]; q[i] = qa[i] + qb[i]; }
  }

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
}

template <int K, int NJ, int NW>
void launch_one(const QuantArgs& a, int total, hipStream_t s) {
  hipLaunchKernelGGL((quantize_kernel<K, NJ, NW>), dim3(total), dim3(64 * NW), 0, s, a);
}

// Waves per vector: one when there are enough vectors to fill the chip (throughput regime),
// 4 or 16 when there are few (latency regime); then the smallest register bucket that holds
// the vector's share.
template <int K>
hipError_t launch_k(const QuantArgs& a, int max_n, hipStream_t s) {
  const int total = a.seg[0].count + a.seg[1].count;
  if (total == 0) return hipSuccess;
  const int nslots = 2 * ((max_n + 127) / 128);
  int nw = total >= 1024 ? 1 : (total >= 96 ? 4 : 16);
  while (nw > 1 && nw > nslots) nw /= 4;
  if (nw == 1 && nslots > 64) nw = 4;
  if (nw == 4 && nslots > 256) return hipErrorInvalidValue;
  const int nj = (nslots + nw - 1) / nw;
  if (nw == 1) {
    if (nj <= 4) launch_one<K, 4, 1>(a, total, s);
    else if (nj <= 16) launch_one<K, 16, 1>(a, total, s);
    else launch_one<K, 64, 1>(a, total, s);
  } else if (nw == 4) {
    if (nj <= 1) launch_one<K, 1, 4>(a, total, s);
    else if (nj <= 4) launch_one<K, 4, 4>(a, total, s);
    else if (nj <= 16) launch_one<K, 16, 4>(a, total, s);
    else launch_one<K, 64, 4>(a, total, s);
  } else {
    if (nj <= 1) launch_one<K, 1, 16>(a, total, s);
    else if (nj <= 4) launch_one<K, 4, 16>(a, total, s);
    else launch_one<K, 16, 16>(a, total, s);
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
