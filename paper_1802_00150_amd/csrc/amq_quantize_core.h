// Device-side core of the alternating multi-bit quantizer (Alg. 2), shared by the stand-alone
// quantizer kernels and the persistent recurrent kernel.  gfx950, 64-wide wavefronts.
//
// Element layout in a wave: "slot" j of a lane holds entry (slot_base + j) * 64 + lane, so a
// wave-wide comparison yields, through the 64-bit ballot, exactly two packed code words of
// the exchange format.  Lane j keeps the ballot of slot j; the Gram matrix of Eq. 5 is then a
// per-lane popcount of xor-ed masks plus one reduction, and the final store of a plane is one
// coalesced 8-byte-per-lane write.
//
// Precision: stored quantities are binary32; the reductions (sum |r|, B^T w) are accumulated
// in binary64 and the k x k system is solved in binary64 with exact integer cofactors, then
// rounded once.  The comparison "w >= midpoint" that decides a code is binary32.
#pragma once
#include "amq_device.h"

namespace amq {

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

// The arithmetic of Alg. 2 for one vector held in registers: `w[j]` of lane L is entry
// (base + j) * 64 + L (0 beyond n); NW waves cooperate (nj slots each).  On return alpha holds the
// coefficients and lane j of each wave holds in mym[i] the 64 packed codes of its slot j of
// plane i.  Stages are selected by the caller: greedy initialisation, then `iters` cycles of
// { Eq. 5 if do_ls; code table + Alg. 1 if do_bst }.  With do_greedy false the caller
// provides alpha, and (if do_ls) mym and the per-lane partial sums q of B^T w.
template <int K, int NJ, int NW>
__device__ __forceinline__ void quantize_core(const float (&w)[NJ], int n, int base, int nj, bool do_greedy,
                                              int iters, bool do_ls, bool do_bst, float (&alpha)[K],
                                              unsigned long long (&mym)[K], double (&q)[K],
                                              double (*sh)[16 * kMaxRed], int& phase) {
  constexpr int M = 1 << K;
  constexpr int NP = K * (K - 1) / 2;
  const int lane = lane_id();
  const double dn = (double)n;
  if (do_greedy) {
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
  }
  for (int it = 0; it < iters; ++it) {
    if (do_ls) {
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
      if (!do_bst) break;
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
    const bool more = do_ls && (it + 1 < iters);  // B^T w is needed by another cycle
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

}

}  // namespace amq
