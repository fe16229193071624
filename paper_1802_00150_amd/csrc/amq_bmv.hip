// Small-batch binary matrix-vector products with the weight planes held in registers and the
// epilogue fused: plain output (streaming GEMV), LSTM cell (Eq. 6) or GRU cell.
//
// Mapping (gfx950, wave64): a weight row of one plane is cpr = wpr/4 16-byte chunks.  A wave
// is split into groups of G = 2^lg lanes (G >= cpr, at most 64); a group owns R = 64/G
// consecutive rows (or hidden units), a lane one chunk.  One wave-wide dwordx4 load therefore
// reads up to 1 KiB of contiguous plane memory.  A wave loads, up front, NSEG row segments
// (gate blocks, or consecutive row groups when streaming) x NBLK operand blocks (x and h) x
// KW planes -- all loads in flight before the first use -- and then loops over the batch with
// the activation planes staged in LDS.  Per batch entry a lane forms the float partial
//   sum_i alpha_i * sum_j beta_j * (bits_in_chunk - 2 * popcount(w_i xor x_j))
// and the G lanes of a group are summed with DPP butterflies (one value per segment instead of
// KW*KA integers).  Lane 0 of the group applies bias / cell nonlinearity and stores.
#include <type_traits>

#include "amq_device.h"
#include "amq_launch.h"

namespace amq {

namespace {

// LSE (store mode only): also leave, per batch entry and wave, the (max, sum of exponentials) of
// the outputs the wave produced, for a log-softmax over the rows that follows.
template <int KW, int KA, int NSEG, int NBLK, int EPI, bool LSE = false>
__global__ __launch_bounds__(256) void bmv_kernel(BmvArgs a) {
  extern __shared__ uint4 xs[];
  const int lane = lane_id(), wv = wave_id();
  const int lg = a.lg;
  const int G = 1 << lg, R = 64 >> lg;
  const int sub = lane & (G - 1), rloc = lane >> lg;
  const long long wave_global = (long long)blockIdx.x * 4 + wv;
  const long long grp = blockIdx.y;
  const int batch = a.batch;

  int cpr[NBLK], xoff[NBLK], bits[NBLK];
  {
    int off = 0;
#pragma unroll
    for (int k = 0; k < NBLK; ++k) {
      const int n = a.blk[k].n;
      cpr[k] = (n + 127) >> 7;
      xoff[k] = off;
      off += KA * batch * cpr[k];
      const int left = n - 128 * sub;
      bits[k] = left < 0 ? 0 : (left > 128 ? 128 : left);
    }
  }

  // rows of this lane: segment s covers rows seg_base(s) + [0, R)
  const long long nrow = (EPI == kEpiStore) ? a.m : a.H;  // rows per segment space
  long long row[NSEG];
  bool ok[NSEG];
#pragma unroll
  for (int s = 0; s < NSEG; ++s) {
    long long r;
    if (EPI == kEpiStore) {
      r = (wave_global * NSEG + s) * R + rloc;
      ok[s] = r < a.m;
    } else {
      const long long u = wave_global * R + rloc;
      ok[s] = u < a.H;
      r = (long long)s * a.H + u;
    }
    row[s] = ok[s] ? r : 0;
  }

  // weight planes and coefficients first: the longest loads go out before anything waits.  Planes that
  // are read once (more of them than the caches hold) are loaded non-temporal: measured on 512 MiB of
  // planes, 6.3 against 5.95 TB/s for the plain product and 4.95 against 4.63 TB/s for the LSTM step.
  uint4 wq[NBLK][NSEG][KW];
  float al[NBLK][NSEG][KW];
  auto request_weights = [&](auto streaming) {
#pragma unroll
    for (int k = 0; k < NBLK; ++k) {
      const int wpr = cpr[k] * 4;
      const uint32_t* Wp = a.blk[k].Wp + grp * (k ? a.g_Wp1 : a.g_Wp);
      const float* alpha = a.blk[k].alpha + grp * (k ? a.g_alpha1 : a.g_alpha);
#pragma unroll
      for (int s = 0; s < NSEG; ++s)
#pragma unroll
        for (int i = 0; i < KW; ++i) {
          const uint4* src = reinterpret_cast<const uint4*>(Wp + ((long long)i * a.m + row[s]) * wpr) + sub;
          if (sub < cpr[k]) wq[k][s][i] = decltype(streaming)::value ? load_streaming(src) : *src;
          else wq[k][s][i] = make_uint4(0, 0, 0, 0);
          al[k][s][i] = alpha[row[s] * KW + i];
        }
    }
  };
  if (a.streaming) request_weights(std::true_type{});
  else request_weights(std::false_type{});
  // biases of this lane's rows (loop-invariant over the batch)
  float bs0[NSEG], bs1[NSEG];
#pragma unroll
  for (int s = 0; s < NSEG; ++s) {
    bs0[s] = a.bias0 ? a.bias0[row[s]] : 0.0f;
    bs1[s] = (EPI == kEpiGru && a.bias1) ? a.bias1[row[s]] : 0.0f;
  }

  // activation planes of every batch entry into LDS
#pragma unroll
  for (int k = 0; k < NBLK; ++k) {
    const int total = KA * batch * cpr[k];
    const uint4* src = reinterpret_cast<const uint4*>(a.blk[k].Xp + grp * (k ? a.g_Xp1 : a.g_Xp));
    for (int t = threadIdx.x; t < total; t += 256) xs[xoff[k] + t] = src[t];
  }
  __syncthreads();
  {
    const long long first = (EPI == kEpiStore) ? wave_global * NSEG * R : wave_global * R;
    if (first >= nrow) return;  // whole wave past the end (after the barrier)
  }

  float* const lse_part = LSE ? a.lse_part : nullptr;  // read once, not per batch entry
  const int lse_slots = a.lse_slots;
  for (int b = 0; b < batch; ++b) {
    // previous state / old output of this batch entry, requested before the popcount work
    float prev[NSEG];
#pragma unroll
    for (int s = 0; s < NSEG; ++s) prev[s] = 0.0f;
    if (sub == 0) {
      if constexpr (EPI == kEpiStore) {
        if (a.accumulate) {
#pragma unroll
          for (int s = 0; s < NSEG; ++s)
            if (ok[s]) prev[s] = a.Y[grp * a.g_Y + (long long)b * a.m + row[s]];
        }
      } else if (ok[0]) {
        prev[0] = (EPI == kEpiLstm) ? a.c_prev[grp * a.g_state + (long long)b * a.H + row[0]]
                                    : a.h_prev[(long long)b * a.H + row[0]];
      }
    }
    float part[NBLK][NSEG];
#pragma unroll
    for (int k = 0; k < NBLK; ++k) {
      uint4 xq[KA];
      float bt[KA];
      const float* beta = a.blk[k].beta + grp * (k ? a.g_beta1 : a.g_beta);
#pragma unroll
      for (int j = 0; j < KA; ++j) {
        xq[j] = (sub < cpr[k]) ? xs[xoff[k] + (j * batch + b) * cpr[k] + sub] : make_uint4(0, 0, 0, 0);
        bt[j] = beta[b * KA + j];
      }
#pragma unroll
      for (int s = 0; s < NSEG; ++s) {
        float acc = 0.0f;
#pragma unroll
        for (int i = 0; i < KW; ++i) {
          float inner = 0.0f;
#pragma unroll
          for (int j = 0; j < KA; ++j)
            inner = fmaf(bt[j], (float)(bits[k] - 2 * popc4(wq[k][s][i], xq[j])), inner);
          acc = fmaf(al[k][s][i], inner, acc);
        }
        part[k][s] = acc;
      }
    }

    if constexpr (EPI == kEpiStore) {
      float yv[NSEG];
#pragma unroll
      for (int s = 0; s < NSEG; ++s) {
        yv[s] = group_sum(part[0][s], lg) + bs0[s] + prev[s];
        if (sub == 0 && ok[s]) a.Y[grp * a.g_Y + (long long)b * a.m + row[s]] = yv[s];
      }
      if constexpr (LSE) {  // (max, sum of exponentials) over this wave's outputs
        float pm = kLseLow, ps = 0.0f;
#pragma unroll
        for (int s = 0; s < NSEG; ++s)
          if (sub == 0 && ok[s]) lse_merge(pm, ps, yv[s], 1.0f);
        lse_wave_merge(pm, ps);
        if (lane == 0) {
          float* dst = lse_part + ((long long)b * lse_slots + wave_global) * 2;
          dst[0] = pm;
          dst[1] = ps;
        }
      }
    } else if constexpr (EPI == kEpiLstm) {
      float pre[4];
#pragma unroll
      for (int s = 0; s < 4; ++s) pre[s] = group_sum(part[0][s] + part[1][s], lg);
      if (sub == 0 && ok[0]) {
        const long long u = row[0];
#pragma unroll
        for (int s = 0; s < 4; ++s) pre[s] += bs0[s];
        const long long t = grp * a.g_state + (long long)b * a.H + u;
        const float gi = sigmoidf_dev(pre[0]);
        const float gf = sigmoidf_dev(pre[1]);
        const float go = sigmoidf_dev(pre[2]);
        const float gg = tanhf_dev(pre[3]);
        const float c = fmaf(gf, prev[0], gi * gg);
        const float h = go * tanhf_dev(c);
        a.c_out[t] = c;
        a.h_out[t] = h;
        if (a.hs_out) a.hs_out[t] = h;
      }
    } else {  // GRU: segments r, z, n; the candidate keeps its x-side and h-side sums apart
      const float sr = group_sum(part[0][0] + part[1][0], lg);
      const float sz = group_sum(part[0][1] + part[1][1], lg);
      const float nx = group_sum(part[0][2], lg);
      const float nh = group_sum(part[1][2], lg);
      if (sub == 0 && ok[0]) {
        const long long t = (long long)b * a.H + row[0];
        const float r = sigmoidf_dev(sr + bs0[0] + bs1[0]);
        const float z = sigmoidf_dev(sz + bs0[1] + bs1[1]);
        const float nn = tanhf_dev(fmaf(r, nh + bs1[2], nx + bs0[2]));
        a.h_out[t] = fmaf(z, prev[0] - nn, nn);
      }
    }
  }
}

template <int KW, int KA, int NSEG, int NBLK, int EPI>
hipError_t launch_one(BmvArgs a, long long waves, size_t lds, hipStream_t s, int* lse_slots) {
  const long long blocks = (waves + 3) / 4;
  const dim3 grid((unsigned)blocks, (unsigned)a.groups);
  // every wave that owns at least one row fills one slot per batch entry
  if (a.lse_part && (waves > kLseMaxSlots || waves > a.lse_cap || a.groups != 1)) a.lse_part = nullptr;
  a.lse_slots = (int)waves;
  if (lse_slots) *lse_slots = a.lse_part ? (int)waves : 0;
  if constexpr (EPI == kEpiStore) {
    if (a.lse_part) {
      hipLaunchKernelGGL((bmv_kernel<KW, KA, NSEG, NBLK, EPI, true>), grid, dim3(256), lds, s, a);
      return hipGetLastError();
    }
  }
  hipLaunchKernelGGL((bmv_kernel<KW, KA, NSEG, NBLK, EPI, false>), grid, dim3(256), lds, s, a);
  return hipGetLastError();
}

template <int KW, int KA>
hipError_t launch_epi(const BmvArgs& a, int epi, hipStream_t s, int* lse_slots) {
  const int R = 64 >> a.lg;
  size_t lds = 0;
  const int nblk = (epi == kEpiStore) ? 1 : 2;
  for (int k = 0; k < nblk; ++k) lds += (size_t)KA * a.batch * ((a.blk[k].n + 127) / 128) * 16;
  switch (epi) {
    case kEpiStore: {
      // four row groups per wave (all loads in flight) when there are enough rows to fill the
      // chip that way; one row group per wave for small products, where parallelism matters more
      const long long waves4 = (a.m + 4LL * R - 1) / (4LL * R);
      if (waves4 * a.groups >= 2048) return launch_one<KW, KA, 4, 1, kEpiStore>(a, waves4, lds, s, lse_slots);
      return launch_one<KW, KA, 1, 1, kEpiStore>(a, (a.m + R - 1) / R, lds, s, lse_slots);
    }
    case kEpiLstm: return launch_one<KW, KA, 4, 2, kEpiLstm>(a, (a.H + R - 1) / R, lds, s, nullptr);
    case kEpiGru: return launch_one<KW, KA, 3, 2, kEpiGru>(a, (a.H + R - 1) / R, lds, s, nullptr);
  }
  return hipErrorInvalidValue;
}

template <int KW>
hipError_t launch_ka(const BmvArgs& a, int k_a, int epi, hipStream_t s, int* lse_slots) {
  switch (k_a) {
    case 1: return launch_epi<KW, 1>(a, epi, s, lse_slots);
    case 2: return launch_epi<KW, 2>(a, epi, s, lse_slots);
    case 3: return launch_epi<KW, 3>(a, epi, s, lse_slots);
    case 4: return launch_epi<KW, 4>(a, epi, s, lse_slots);
  }
  return hipErrorInvalidValue;
}

}  // namespace

bool bmv_supported(int n0, int n1, int k_a, long long batch, int epi) {
  const int c0 = (n0 + 127) / 128, c1 = (n1 + 127) / 128;
  const bool fp4 = n0 <= 1024 && n1 <= 1024;  // the fp4 matrix-core kernels are the alternative
  const int limit = !fp4 ? kBmvMaxBatch : epi == kEpiStore ? kBmvMaxBatchStore : kBmvMaxBatchCell;
  if (c0 > 64 || c1 > 64 || batch > limit) return false;
  return (size_t)k_a * batch * (c0 + c1) * 16 <= 48 * 1024;
}

hipError_t launch_bmv(BmvArgs a, int k_w, int k_a, int epi, hipStream_t s, int* lse_slots) {
  if (lse_slots) *lse_slots = 0;
  if (epi != kEpiStore) a.lse_part = nullptr;
  int nmax = a.blk[0].n;
  if (epi != kEpiStore && a.blk[1].n > nmax) nmax = a.blk[1].n;
  const int cpr = (nmax + 127) / 128;
  int lg = 0;
  while ((1 << lg) < cpr) ++lg;
  a.lg = lg;
  {
    long long plane_bytes = (long long)k_w * a.m * ((a.blk[0].n + 127) / 128) * 16;
    if (epi != kEpiStore) plane_bytes += (long long)k_w * a.m * ((a.blk[1].n + 127) / 128) * 16;
    a.streaming = plane_bytes * a.groups > kBmvStreamingBytes;
  }
  switch (k_w) {
    case 1: return launch_ka<1>(a, k_a, epi, s, lse_slots);
    case 2: return launch_ka<2>(a, k_a, epi, s, lse_slots);
    case 3: return launch_ka<3>(a, k_a, epi, s, lse_slots);
    case 4: return launch_ka<4>(a, k_a, epi, s, lse_slots);
  }
  return hipErrorInvalidValue;
}

}  // namespace amq
