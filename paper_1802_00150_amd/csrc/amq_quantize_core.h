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
#include <type_traits>

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

// 1 / d for an integer-valued d != 0 far from the ends of the exponent range: hardware estimate
// and two Newton steps (error below one unit in the last place of binary64, which disappears when
// the coefficients are rounded to binary32).
__device__ __forceinline__ double recip_f64(double d) {
  double r = __builtin_amdgcn_rcp(d);
  r = __builtin_fma(r, __builtin_fma(-d, r, 1.0), r);
  r = __builtin_fma(r, __builtin_fma(-d, r, 1.0), r);
  return r;
}

// Eq. 5 on the vector unit in binary64 for K <= 3, from the disagreement counts d[t] of the plane
// pairs (order (0,1), (0,2), (1,2)): G_ij = n - 2 d_ij, cofactors and determinant are integers below
// 2^45 for n <= 16384 and therefore exact in binary64 (same values as the integer cofactors of
// ls_solve); alpha_i = (sum_j cof_ji q_j) / det.  A singular G leaves alpha unchanged.
template <int K>
__device__ __forceinline__ void ls_solve_f64(int n, const double* d, const double (&q)[K], float (&alpha)[K]) {
  static_assert(K >= 1 && K <= 3, "binary64 cofactors are exact up to K = 3");
  const double dn = (double)n;
  if constexpr (K == 1) {
    alpha[0] = (float)(q[0] / dn);
  } else if constexpr (K == 2) {
    const double a = dn - 2.0 * d[0];
    const double det = dn * dn - a * a;
    if (det == 0.0) return;
    const double inv = recip_f64(det);
    alpha[0] = (float)((dn * q[0] + (-a) * q[1]) * inv);
    alpha[1] = (float)(((-a) * q[0] + dn * q[1]) * inv);
  } else {
    const double a = dn - 2.0 * d[0], b = dn - 2.0 * d[1], c = dn - 2.0 * d[2];
    const double nn = dn * dn;
    const double c00 = nn - c * c, c01 = c * b - a * dn, c02 = a * c - dn * b;
    const double c11 = nn - b * b, c12 = a * b - dn * c, c22 = nn - a * a;
    const double det = dn * c00 + a * c01 + b * c02;
    if (det == 0.0) return;
    const double inv = recip_f64(det);
    alpha[0] = (float)((c00 * q[0] + c01 * q[1] + c02 * q[2]) * inv);
    alpha[1] = (float)((c01 * q[0] + c11 * q[1] + c12 * q[2]) * inv);
    alpha[2] = (float)((c02 * q[0] + c12 * q[1] + c22 * q[2]) * inv);
  }
}

// v_writelane_b32: lane `lane` (a constant) of `old` takes the wave-uniform `value`.  (The compiler's
// intrinsic, reached by its name: this compiler has no builtin for it.)
extern "C" __device__ int amq_writelane_i32(int value, int lane, int old) __asm("llvm.amdgcn.writelane.i32");

// This lane's bit of a wave-uniform 64-bit mask, as a condition (the mask becomes the lane mask of whatever
// selects on it; no vector instruction).
extern "C" __device__ bool amq_inverse_ballot_i64(unsigned long long mask) __asm("llvm.amdgcn.inverse.ballot.i64");
__device__ __forceinline__ bool lane_bit(unsigned long long mask) { return amq_inverse_ballot_i64(mask); }

// Up to this many planes the code assignment of the throughput path works on comparison masks (scalar
// unit); beyond, the 2^K - 1 masks and the logic on them cost more than counting the comparisons per lane
// (measured at K = 3 on 16384 x 4096: 320 us with mask logic, 264 us with counted comparisons).
constexpr int kMaskLogicMaxK = 2;

// Lane j keeps the wave-uniform 64-bit value `mk` (the ballot of slot j): one lane write per half, which
// takes the value straight from the scalar registers the comparison wrote.
__device__ __forceinline__ void keep_in_lane(unsigned long long& mine, unsigned long long mk, int j) {
  int lo = (int)(unsigned)(mine & 0xffffffffull), hi = (int)(unsigned)(mine >> 32);
  lo = amq_writelane_i32((int)(unsigned)(mk & 0xffffffffull), j, lo);
  hi = amq_writelane_i32((int)(unsigned)(mk >> 32), j, hi);
  mine = ((unsigned long long)(unsigned)hi << 32) | (unsigned)lo;
}

__device__ __forceinline__ float readlane_f(float v, int l) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l));
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_d(double v) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  if constexpr (ROW_MASK == 0xf) {
    // every lane is written from a valid lane: no previous value to keep, no register to clear
    lo = __builtin_amdgcn_update_dpp(0, lo, CTRL, 0xf, 0xf, true);
    hi = __builtin_amdgcn_update_dpp(0, hi, CTRL, 0xf, 0xf, true);
  } else {
    lo = __builtin_amdgcn_update_dpp(0, lo, CTRL, ROW_MASK, 0xf, false);
    hi = __builtin_amdgcn_update_dpp(0, hi, CTRL, ROW_MASK, 0xf, false);
  }
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

// Totals over the workgroup of NQ per-lane doubles q and of NC values c that are already totals of
// their wave (wave-uniform); results in q and c.  One LDS barrier.
template <int NW, int NQ, int NC>
__device__ __forceinline__ void block_totals_mixed(double (&q)[NQ], double (&c)[NC > 0 ? NC : 1],
                                                   double (*sh)[16 * kMaxRed], int& phase) {
  wave_totals<NQ>(q);
  if constexpr (NW > 1) {
    const int wv = wave_id();
    if (lane_id() == 0) {
#pragma unroll
      for (int i = 0; i < NQ; ++i) sh[phase][wv * (NQ + NC) + i] = q[i];
#pragma unroll
      for (int i = 0; i < NC; ++i) sh[phase][wv * (NQ + NC) + NQ + i] = c[i];
    }
    lds_barrier();
#pragma unroll
    for (int i = 0; i < NQ + NC; ++i) {
      double t = sh[phase][i];
#pragma unroll
      for (int w = 1; w < NW; ++w) t += sh[phase][w * (NQ + NC) + i];
      if (i < NQ) q[i] = t; else c[i - NQ] = t;
    }
    phase ^= 1;
  }
}

// Alg. 2 for one vector of at most 4 slots per lane, tuned for the latency of a single vector (the
// on-line case): the codes of a slot are kept as wave-uniform 64-bit ballots (scalar registers), so
// the disagreement counts of Eq. 5 are scalar popcounts with no cross-lane reduction, only B^T w
// travels through the binary64 lane reduction, and the K x K system is solved in binary64 on the
// vector unit (K <= 3).  Same interface and results as quantize_core below.
template <int K, int NJ, int NW>
__device__ __forceinline__ void quantize_core_uniform(const float (&w)[NJ], int n, int base, int nj, bool do_greedy,
                                                      int iters, bool do_ls, bool do_bst, float (&alpha)[K],
                                                      unsigned long long (&mym)[K], double (&q)[K],
                                                      double (*sh)[16 * kMaxRed], int& phase,
                                                      unsigned long long* marks) {
  (void)marks;
  static_assert(NJ <= 4, "ballots of every slot and plane live in scalar registers");
  constexpr int M = 1 << K;
  constexpr int NP = K * (K - 1) / 2;
  const int lane = lane_id();
  const double dn = (double)n;
  const bool n_pow2 = (n & (n - 1)) == 0;
  const double inv_n = 1.0 / dn;  // exact for a power of two, where s / n == s * inv_n bit for bit
  unsigned long long mk[K][NJ];   // mk[i][j]: plane i of slot j, bit = lane
#pragma unroll
  for (int i = 0; i < K; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) mk[i][j] = 0ull;
  // Which lanes of a slot lie inside the vector, as wave-uniform masks.  A comparison is written so that its
  // ballot is the comparison's own scalar result, and "inside the vector" is an AND on the scalar unit;
  // where a lane needs a mask as a condition it takes its bit straight from the mask (lane_bit).  A wave
  // whose slots all lie inside (the usual case: 1024 entries on four waves) runs a form without the masks.
  unsigned long long inside[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) inside[j] = (j < nj) ? __ballot((base + j) * 64 + lane < n) : 0ull;
  const bool all_inside = nj == NJ && (base + NJ) * 64 <= n;
  double wd[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) wd[j] = (double)w[j];

  auto greedy = [&](auto full_c) {
    constexpr bool FULL = decltype(full_c)::value;
    // ---- greedy initialisation, Eq. 4 (one pass per stage, as in quantize_core)
    float r[NJ];
    double s[1];
    double lane_l1;  // this lane's share of sum |w|, which is also its share of b_1^T w (same terms, same order)
    {
      double s0 = 0.0, s1 = 0.0;
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        r[j] = w[j];
        if (j & 1) s1 += (double)fabsf(w[j]); else s0 += (double)fabsf(w[j]);
      }
      lane_l1 = s0 + s1;
      s[0] = lane_l1;
    }
    block_totals<NW, 1>(s, sh, phase);
#pragma unroll
    for (int i = 0; i < K; ++i) {
      const float al = n_pow2 ? (float)(s[0] * inv_n) : (float)(s[0] / dn);
      alpha[i] = al;
      // (sums of +-w start from their first term: 0.0 + x is an instruction the compiler may not drop,
      // x being -0.0 for all it knows)
      double q0 = 0.0, q1 = 0.0, s0 = 0.0, s1 = 0.0;
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const unsigned long long ge = __ballot(r[j] >= 0.0f);
        const unsigned long long m = FULL ? ge : (ge & inside[j]);
        mk[i][j] = m;
        const bool bit = lane_bit(m);
        if constexpr (K > 1) {
          float rn = r[j] - (bit ? al : -al);
          if constexpr (!FULL) rn = lane_bit(inside[j]) ? rn : 0.0f;
          r[j] = rn;
          if (i > 0) {
            const double sw = bit ? wd[j] : -wd[j];
            if (j & 1) q1 = (j == 1) ? sw : q1 + sw; else q0 = (j == 0) ? sw : q0 + sw;
          }
          if (i + 1 < K) {
            if (j & 1) s1 += (double)fabsf(rn); else s0 += (double)fabsf(rn);
          }
        }
      }
      q[i] = (i == 0) ? lane_l1 : (NJ > 1 ? q0 + q1 : q0);
      if (i + 1 < K) {
        s[0] = s0 + s1;
        block_totals<NW, 1>(s, sh, phase);
      }
    }
  };
  if (do_greedy) {
    if (all_inside) greedy(std::true_type{}); else greedy(std::false_type{});
  } else if (do_ls) {
    // codes given by the caller as per-lane masks (lane j holds slot j)
#pragma unroll
    for (int i = 0; i < K; ++i) {
      const int lo = (int)(mym[i] & 0xffffffffull), hi = (int)(mym[i] >> 32);
#pragma unroll
      for (int j = 0; j < NJ; ++j)
        mk[i][j] = ((unsigned long long)(unsigned)__builtin_amdgcn_readlane(hi, j) << 32) |
                   (unsigned)__builtin_amdgcn_readlane(lo, j);
    }
  }
  AMQ_PHASE(marks, 2);
  for (int it = 0; it < iters; ++it) {
    if (do_ls) {
      // ---- Eq. 5: B^T w through the lane reduction, the disagreement counts of the plane pairs
      // from the ballots on the scalar unit
      double cnt[NP > 0 ? NP : 1];
      {
        int t = 0;
#pragma unroll
        for (int a = 0; a < K; ++a)
#pragma unroll
          for (int b = a + 1; b < K; ++b) {
            int c = 0;
#pragma unroll
            for (int j = 0; j < NJ; ++j) c += __popcll(mk[a][j] ^ mk[b][j]);
            cnt[t++] = (double)c;
          }
      }
      block_totals_mixed<NW, K, NP>(q, cnt, sh, phase);
      AMQ_PHASE(marks, 4 + 4 * it);
      if constexpr (K <= 3) {
        ls_solve_f64<K>(n, cnt, q, alpha);
      } else {
        int G[K][K];
        int t = 0;
#pragma unroll
        for (int a = 0; a < K; ++a) {
          G[a][a] = n;
#pragma unroll
          for (int b = a + 1; b < K; ++b) {
            const int d = __builtin_amdgcn_readfirstlane((int)cnt[t++]);
            G[a][b] = n - 2 * d;
            G[b][a] = G[a][b];
          }
        }
        ls_solve<K>(G, q, alpha);
      }
      AMQ_PHASE(marks, 5 + 4 * it);
      if (!do_bst) break;
    }

    // ---- code table in ascending order (Alg. 2), across lanes as in quantize_core
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
    // midpoint of a code and its upper neighbour: every lane forms its own (the neighbour's value comes
    // through a row shift), the first M - 1 are then read out as wave-uniform values
    const float up = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(sv), 0x101 /* row_shl:1 */, 0xf, 0xf, true));
    const float mid = 0.5f * (sv + up);
    float thr[M - 1];
#pragma unroll
    for (int j = 0; j < M - 1; ++j) thr[j] = readlane_f(mid, j);
    unsigned bm[K];  // bit `pos` of bm[i]: plane i is +1 for the code at sorted position pos
#pragma unroll
    for (int i = 0; i < K; ++i) bm[i] = (unsigned)__ballot((sp & (1 << (K - 1 - i))) != 0) & (unsigned)((1ull << M) - 1ull);
    AMQ_PHASE(marks, 6 + 4 * it);

    // ---- codes with the coefficients fixed (Alg. 1)
    const bool more = do_ls && (it + 1 < iters);
    auto assign = [&](auto full_c, auto more_c) {
      constexpr bool FULL = decltype(full_c)::value;
      constexpr bool MORE = decltype(more_c)::value;  // B^T w is needed by another cycle
      double qa[K], qb[K];
#pragma unroll
      for (int i = 0; i < K; ++i) { qa[i] = 0.0; qb[i] = 0.0; }
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        int pos = 0;  // position in the sorted table = number of midpoints <= w
#pragma unroll
        for (int t = 0; t < M - 1; ++t) pos += (w[j] >= thr[t]) ? 1 : 0;
        const unsigned sel = 1u << pos;
#pragma unroll
        for (int i = 0; i < K; ++i) {
          const unsigned long long hit = __ballot((sel & bm[i]) != 0u);
          const unsigned long long m = FULL ? hit : (hit & inside[j]);
          mk[i][j] = m;
          if constexpr (MORE) {
            const double sw = lane_bit(m) ? wd[j] : -wd[j];
            if (j & 1) qb[i] = (j == 1) ? sw : qb[i] + sw; else qa[i] = (j == 0) ? sw : qa[i] + sw;
          }
        }
      }
      if constexpr (MORE) {
#pragma unroll
        for (int i = 0; i < K; ++i) q[i] = NJ > 1 ? qa[i] + qb[i] : qa[i];
      }
    };
    if (all_inside) {
      if (more) assign(std::true_type{}, std::true_type{}); else assign(std::true_type{}, std::false_type{});
    } else {
      if (more) assign(std::false_type{}, std::true_type{}); else assign(std::false_type{}, std::false_type{});
    }
    AMQ_PHASE(marks, 7 + 4 * it);
  }
  // lane j takes the ballots of slot j (the layout the callers store)
#pragma unroll
  for (int i = 0; i < K; ++i) {
    unsigned long long mine = 0ull;
#pragma unroll
    for (int j = 0; j < NJ; ++j) keep_in_lane(mine, mk[i][j], j);
    mym[i] = mine;
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
                                              double (*sh)[16 * kMaxRed], int& phase,
                                              unsigned long long* marks = nullptr) {
  (void)marks;  // phase timers of the profiling build: 2 = greedy done, 4 + 4 * cycle + {0: reduction, 1: solve, 2: table, 3: assignment}
  if constexpr (NJ <= 4 && K <= 3) {  // (K = 4 would need more scalar registers than a wave has)
    quantize_core_uniform<K, NJ, NW>(w, n, base, nj, do_greedy, iters, do_ls, do_bst, alpha, mym, q, sh, phase, marks);
    return;
  }
  constexpr int M = 1 << K;
  constexpr int NP = K * (K - 1) / 2;
  const int lane = lane_id();
  const double dn = (double)n;
  const bool n_pow2 = (n & (n - 1)) == 0;
  const double inv_n = 1.0 / dn;  // exact for a power of two, where s / n == s * inv_n bit for bit
  // Every slot of this wave inside the vector (the common case of the throughput regime: rows whose
  // length is a multiple of 64 * NJ * NW) takes a second instantiation of the per-entry loops without
  // the range checks.
  const bool full = nj == NJ && (base + NJ) * 64 <= n;
  // One cycle has no effect at K = 1 (Eq. 5 returns sum |w| / n again -- the same terms in the same
  // order -- and the only midpoint of the code table {-alpha, +alpha} is 0), so the greedy codes and
  // coefficient are final there.
  if (K == 1 && do_greedy) iters = 0;

  auto greedy = [&](auto full_c) {
    constexpr bool FULL = decltype(full_c)::value;
    // ---- greedy initialisation, Eq. 4.  One pass per stage: it assigns the signs, updates the
    // residual and accumulates the l1 norm of the new residual for the next stage.
    float r[NJ];
    double s[1];
    double lane_l1;  // this lane's share of sum |w|, which is also its share of b_1^T w
    {
      double s0 = 0.0, s1 = 0.0;
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        r[j] = w[j];
        if (j & 1) s1 += (double)fabsf(w[j]); else s0 += (double)fabsf(w[j]);
      }
      lane_l1 = s0 + s1;
      s[0] = lane_l1;
    }
    block_totals<NW, 1>(s, sh, phase);
#pragma unroll
    for (int i = 0; i < K; ++i) {
      const float al = n_pow2 ? (float)(s[0] * inv_n) : (float)(s[0] / dn);
      alpha[i] = al;
      unsigned long long mine = 0ull;
      double q0 = 0.0, q1 = 0.0, s0 = 0.0, s1 = 0.0;
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        if (FULL || j < nj) {
          const bool valid = FULL || (base + j) * 64 + lane < n;
          const bool bit = valid && (r[j] >= 0.0f);
          keep_in_lane(mine, __ballot(bit), j);
          if constexpr (K > 1) {
            const float rn = valid ? r[j] - (bit ? al : -al) : 0.0f;
            r[j] = rn;
            if (i > 0) {  // (stage 0: b_1^T w is sum |w|, term by term)
              const double sw = bit ? (double)w[j] : -(double)w[j];
              if (j & 1) q1 += sw; else q0 += sw;
            }
            if (i + 1 < K) {
              if (j & 1) s1 += (double)fabsf(rn); else s0 += (double)fabsf(rn);
            }
          }
        }
        // (keeps the slots apart: left alone, the scheduler forms all ballots first and spills them)
        if ((j & 3) == 3) __builtin_amdgcn_sched_barrier(0);
      }
      mym[i] = mine;
      q[i] = (i == 0) ? lane_l1 : q0 + q1;
      if (i + 1 < K) {
        s[0] = s0 + s1;
        block_totals<NW, 1>(s, sh, phase);
      }
    }
  };
  if (do_greedy) {
    if (full) greedy(std::true_type{}); else greedy(std::false_type{});
  }
  AMQ_PHASE(marks, 2);
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
      AMQ_PHASE(marks, 4 + 4 * it);
      if constexpr (K <= 3) {
        double qq[K];
#pragma unroll
        for (int i = 0; i < K; ++i) qq[i] = red[i];
        ls_solve_f64<K>(n, red + K, qq, alpha);
      } else {
        int G[K][K];
        double qq[K];
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
        ls_solve<K>(G, qq, alpha);
      }
      AMQ_PHASE(marks, 5 + 4 * it);
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
    AMQ_PHASE(marks, 6 + 4 * it);

    // ---- codes with the coefficients fixed (Alg. 1); the position in the sorted table is the
    // number of midpoints <= w, which is where the k-comparison tree walk ends.
    const bool more = do_ls && (it + 1 < iters);  // B^T w is needed by another cycle
    // wave-uniform masks (all ones or zero): the table's bit at position 0; whether it changes after position t
    unsigned long long first[K], flips[K][M - 1];
#pragma unroll
    for (int i = 0; i < K; ++i) {
      first[i] = 0ull - (unsigned long long)(bm[i] & 1u);
#pragma unroll
      for (int t = 0; t < M - 1; ++t) flips[i][t] = 0ull - (unsigned long long)(((bm[i] >> t) ^ (bm[i] >> (t + 1))) & 1u);
    }
    auto assign = [&](auto full_c, auto more_c) {
      constexpr bool FULL = decltype(full_c)::value;
      constexpr bool MORE = decltype(more_c)::value;
      unsigned long long mine[K];
      double qa[K], qb[K];
#pragma unroll
      for (int i = 0; i < K; ++i) { mine[i] = 0ull; qa[i] = 0.0; qb[i] = 0.0; }
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        if (FULL || j < nj) {
          const bool valid = FULL || (base + j) * 64 + lane < n;
          const double wd = (double)w[j];
          unsigned long long plane[K];  // wave-uniform: plane i of the 64 codes of this slot
          if constexpr (K <= kMaskLogicMaxK) {
            // The comparisons with the ascending midpoints form a thermometer code, so plane i of an
            // entry's code is the table's bit at position 0, flipped once for every midpoint <= w at which
            // the table's bit changes: logic on whole comparison masks, on the scalar unit.
            unsigned long long ge[M - 1];
#pragma unroll
            for (int t = 0; t < M - 1; ++t) ge[t] = __ballot(w[j] >= thr[t]);
            const unsigned long long in_range = FULL ? ~0ull : __ballot(valid);
#pragma unroll
            for (int i = 0; i < K; ++i) {
              unsigned long long b = first[i];
#pragma unroll
              for (int t = 0; t < M - 1; ++t) b ^= ge[t] & flips[i][t];
              plane[i] = FULL ? b : (b & in_range);
            }
          } else {
            int pos = 0;
#pragma unroll
            for (int t = 0; t < M - 1; ++t) pos += (w[j] >= thr[t]) ? 1 : 0;
#pragma unroll
            for (int i = 0; i < K; ++i) plane[i] = __ballot(valid && ((bm[i] >> pos) & 1u));
          }
#pragma unroll
          for (int i = 0; i < K; ++i) {
            keep_in_lane(mine[i], plane[i], j);
            if constexpr (MORE) {
              const bool bit = lane_bit(plane[i]);
              if (j & 1) qb[i] += bit ? wd : -wd; else qa[i] += bit ? wd : -wd;
            }
          }
        }
        if ((j & 3) == 3) __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int i = 0; i < K; ++i) { mym[i] = mine[i]; q[i] = qa[i] + qb[i]; }
    };
    if (full) {
      if (more) assign(std::true_type{}, std::true_type{}); else assign(std::true_type{}, std::false_type{});
    } else {
      if (more) assign(std::false_type{}, std::true_type{}); else assign(std::false_type{}, std::false_type{});
    }
    AMQ_PHASE(marks, 7 + 4 * it);
  }
}

}  // namespace amq
