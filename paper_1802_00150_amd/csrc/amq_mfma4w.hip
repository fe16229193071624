// Large batched binary matrix products on the fp4 matrix cores of gfx950 (Fig. 3 right):
// Y = (sum_i alpha_i B_i)(sum_j beta_j x_j) for many rows and 32 or more columns (mfma4w_kernel),
// and the recurrent steps for batches of 128 and more (mfma4wc_kernel, further down).
//
// Same matrix instruction as the kernel in amq_mfma4.hip (codes as E2M1 nibbles,
// v_mfma_scale_f32_16x16x128_f8f6f4), different work split.  There a wave owns one 16 x 16 output tile
// per pass, and per pass it spends about 350 vector instructions (1400 cycles) on addressing, expanding
// the weight words, popcounts and the coefficient epilogue against k_w k_a 8 matrix instructions (900
// cycles at W2/A3): the vector unit, not the matrix core, bounds it.  Here a wave owns 16 rows x NBT batch
// tiles, so that everything on the weight side (loads, expansion, row coefficients) is paid once per NBT
// tiles and only the per-output epilogue grows with the tile count.  A workgroup of 8 waves stages NBT * 16
// batch entries (all planes) in LDS once and its waves walk over row blocks.  mfma4w_kernel works on
// {-1, +1} codes (the staged activations hold 0.0 beyond the end of a vector), so its accumulators are the
// dot products of the codes and no popcount enters; mfma4wc_kernel still uses {0, 1} codes with popcount
// corrections.
#include <type_traits>

#include "amq_device.h"
#include "amq_launch.h"
#include "amq_pair_body.h"

namespace amq {

namespace {

constexpr int kWaves = 8;

// Contraction of one operand block of a row block with NBT staged batch tiles: units u = (k-step t,
// tile bt); the LDS reads (and, when the step changes, the weight expansion) of unit u + 1 are
// issued under the matrix instructions of unit u.  `tile` points at this lane's 16 bytes of step 0
// of the block's first tile and plane ([tile][plane][kPlaneBytes] layout).
template <int KW, int KA, int NBT, bool SIGNED = false>
__device__ __forceinline__ void contract_tiles(const uint4 (&araw)[KW][2], const unsigned char* tile,
                                               v4f (&acc)[NBT][KW][KA]) {
  // weight words as {0, 1} codes, or as {-1, +1} codes (then the staged tiles are signed too and hold 0.0
  // beyond the end of a vector, and the accumulators are the dot products of the codes themselves)
  auto expand = [](uint32_t w) { return SIGNED ? expand4_signed(w) : expand4(w); };
#pragma unroll
  for (int bt = 0; bt < NBT; ++bt)
#pragma unroll
    for (int i = 0; i < KW; ++i)
#pragma unroll
      for (int j = 0; j < KA; ++j) acc[bt][i][j] = v4f{0.f, 0.f, 0.f, 0.f};
  uint4 bop[KA], bnx[KA], aop[KW], anx[KW];
#pragma unroll
  for (int j = 0; j < KA; ++j) bop[j] = *reinterpret_cast<const uint4*>(tile + j * kPlaneBytes);
#pragma unroll
  for (int i = 0; i < KW; ++i) aop[i] = expand(word_of(araw[i], 0));
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int u = 0; u < kSteps * NBT; ++u) {
    const int bt = u % NBT;
    const int tn = (u + 1) / NBT, bn = (u + 1) % NBT;
    if (u + 1 < kSteps * NBT) {
#pragma unroll
      for (int j = 0; j < KA; ++j)
        bnx[j] = *reinterpret_cast<const uint4*>(tile + (bn * KA + j) * kPlaneBytes + tn * kTileB * 64);
      if (bn == 0) {
#pragma unroll
        for (int i = 0; i < KW; ++i) anx[i] = expand(word_of(araw[i], tn));
      }
    }
#pragma unroll
    for (int i = 0; i < KW; ++i)
#pragma unroll
      for (int j = 0; j < KA; ++j)
        acc[bt][i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(as_operand(aop[i]), as_operand(bop[j]),
                                                                         acc[bt][i][j], 4, 4, 0, kScaleOne, 0, kScaleOne);
    __builtin_amdgcn_sched_group_barrier(0x100, KA, 0);
#pragma unroll
    for (int g = 0; g < KW * KA; ++g) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < KA; ++j) bop[j] = bnx[j];
    if (bn == 0) {
#pragma unroll
      for (int i = 0; i < KW; ++i) aop[i] = anx[i];
    }
  }
  // An MFMA reads its operands from all 64 lanes, but the compiler treats it as lane-local and
  // would sink it into the divergent branches that guard the stores of the epilogues, where lanes
  // of padded batch columns -- which still supply weight rows -- are masked off.  Pin the
  // accumulators here, in uniform control flow.
#pragma unroll
  for (int bt = 0; bt < NBT; ++bt)
#pragma unroll
    for (int i = 0; i < KW; ++i)
#pragma unroll
      for (int j = 0; j < KA; ++j) asm volatile("" : "+v"(acc[bt][i][j]));
}

// Stages the packed activation words of one operand block (NBT * 16 batch entries from bg0 on,
// KA planes) into LDS as 4-bit codes, [tile][plane][step][batch entry][k-block][16 B], and adds
// leaves their popcounts in pops [tile][plane][batch entry].
template <int KA, int NBT, int NTHREADS>
__device__ __forceinline__ void load_activation_words(const uint32_t* Xp, int batch, int bg0, int wq,
                                                      uint4 (&xw)[(NBT * KA * kTileB * 8 + NTHREADS - 1) / NTHREADS]) {
  constexpr int kGroupB = NBT * kTileB;
  constexpr int kItems = NBT * KA * kTileB * 8;
  constexpr int kIter = (kItems + NTHREADS - 1) / NTHREADS;
  const uint4* Xp4 = reinterpret_cast<const uint4*>(Xp);
#pragma unroll
  for (int it = 0; it < kIter; ++it) {
    const int e = threadIdx.x + it * NTHREADS;
    const int q = e & 7, nn = (e >> 3) % kGroupB, j = (e >> 3) / kGroupB;
    const bool valid = e < kItems && bg0 + nn < batch && q < wq;
    const int bb = bg0 + nn < batch ? bg0 + nn : batch - 1;
    const uint4 v = Xp4[((e < kItems ? j : 0) * batch + bb) * wq + (q < wq ? q : 0)];
    xw[it] = valid ? v : make_uint4(0, 0, 0, 0);
  }
}
// SIGNED: {-1, +1} codes with 0.0 at the positions from nlen on (no popcounts are needed then: pops may be
// null).
template <int KA, int NBT, int NTHREADS, bool SIGNED = false>
__device__ __forceinline__ void stage_activation_words(
    const uint4 (&xw)[(NBT * KA * kTileB * 8 + NTHREADS - 1) / NTHREADS], unsigned char* btile, int* pops,
    int nlen = 0) {
  constexpr int kGroupB = NBT * kTileB;
  constexpr int kItems = NBT * KA * kTileB * 8;
  constexpr int kIter = (kItems + NTHREADS - 1) / NTHREADS;
#pragma unroll
  for (int it = 0; it < kIter; ++it) {
    const int e = threadIdx.x + it * NTHREADS;
    const int q = e & 7, nn = (e >> 3) % kGroupB, j = (e >> 3) / kGroupB;
    const int bt = nn >> 4, n16 = nn & 15;
    const uint4 w4 = xw[it];
    // popcount of the row: its 8 groups sit in 8 consecutive lanes (every lane takes part)
    int pc = 0;
    if constexpr (!SIGNED) pc = sum8(__popc(w4.x) + __popc(w4.y) + __popc(w4.z) + __popc(w4.w));
    if (e < kItems) {
      if constexpr (!SIGNED) {
        if (q == 0) pops[(bt * KA + j) * kTileB + n16] = pc;
      }
      // words 4q .. 4q+3 of the row: k-block q >> 1, steps 4 * (q & 1) + 0..3
      uint4* dst = reinterpret_cast<uint4*>(btile + (bt * KA + j) * kPlaneBytes + ((4 * (q & 1)) * kTileB + n16) * 64 +
                                            (q >> 1) * 16);
      if constexpr (SIGNED) {
        // word 4q + c of the row holds positions 32 (4q + c) .. + 31
        auto inside = [&](int c) {
          const int left = nlen - 32 * (4 * q + c);
          return left >= 32 ? 0xffffffffu : left <= 0 ? 0u : ((1u << left) - 1u);
        };
        dst[0 * kTileB * 4] = expand4_signed_valid(w4.x, inside(0));
        dst[1 * kTileB * 4] = expand4_signed_valid(w4.y, inside(1));
        dst[2 * kTileB * 4] = expand4_signed_valid(w4.z, inside(2));
        dst[3 * kTileB * 4] = expand4_signed_valid(w4.w, inside(3));
      } else {
        dst[0 * kTileB * 4] = expand4(w4.x);
        dst[1 * kTileB * 4] = expand4(w4.y);
        dst[2 * kTileB * 4] = expand4(w4.z);
        dst[3 * kTileB * 4] = expand4(w4.w);
      }
    }
  }
}

template <int KW, int KA, int NBT>
__global__ __launch_bounds__(64 * kWaves) void mfma4w_kernel(BmvArgs a, int rb_per_wg, int rowblocks) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int kGroupB = NBT * kTileB;               // batch entries per workgroup
  constexpr int kIter = (NBT * KA * kTileB * 8 + 64 * kWaves - 1) / (64 * kWaves);
  unsigned char* btile = smem;                                           // [tile][plane][kPlaneBytes]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15, l4 = lane >> 4;
  const int bg0 = blockIdx.y * kGroupB;
  const int batch = a.batch;
  const int m = (int)a.m;
  const int nlen = a.blk[0].n;
  const int wq = (nlen + 127) >> 7;  // 16-byte groups per row
  const uint4* Wp4 = reinterpret_cast<const uint4*>(a.blk[0].Wp);
  const float* alpha = a.blk[0].alpha;
  const int rb_first = blockIdx.x * rb_per_wg;
  int rb_end = rb_first + rb_per_wg;
  if (rb_end > rowblocks) rb_end = rowblocks;

  // ---- prologue: packed activation words, 16 bytes per thread and round, coalesced.  Item e:
  // group q = e % 8 of the row of batch entry (e / 8) % kGroupB of plane e / (8 kGroupB).
  {
    uint4 xw[kIter];
    load_activation_words<KA, NBT, 64 * kWaves>(a.blk[0].Xp, batch, bg0, wq, xw);
    stage_activation_words<KA, NBT, 64 * kWaves, true>(xw, btile, nullptr, nlen);
    __syncthreads();
  }

  // coefficients of this lane's batch column, one column per tile
  int bcol[NBT];
  bool bok[NBT];
  float btv[NBT][KA];
#pragma unroll
  for (int bt = 0; bt < NBT; ++bt) {
    bcol[bt] = bg0 + bt * kTileB + l16;
    bok[bt] = bcol[bt] < batch;
    const int bc = bok[bt] ? bcol[bt] : batch - 1;
#pragma unroll
    for (int j = 0; j < KA; ++j) btv[bt][j] = a.blk[0].beta[bc * KA + j];
  }

  // optional: the output row whose value is wanted on its own, per batch column
  long long tg[NBT];
#pragma unroll
  for (int bt = 0; bt < NBT; ++bt) tg[bt] = (a.tgt && bok[bt]) ? a.tgt[bcol[bt]] : -1;

  float lse_m[NBT], lse_s[NBT];  // running (max, sum exp) of this lane's outputs, per tile
#pragma unroll
  for (int bt = 0; bt < NBT; ++bt) {
    lse_m[bt] = kLseLow;
    lse_s[bt] = 0.0f;
  }
  float* const lse_part = a.lse_part;
  const unsigned char* tile = btile + l16 * 64 + l4 * 16;

  // Requests of a row block: its packed weight words in the A-operand view (lane = (tile row l16, k-block
  // l4)) and its row coefficients and bias, one value per lane.  Every request is unconditional on a
  // clamped row (results of rows outside the matrix are masked or never stored), and those of the next row
  // block of this wave go out before the contraction of the current one.
  const int plane = m * wq;
  auto request_rowblock = [&](int rb, uint4 (&raw)[KW][2], float& coef, float& bs) {
    const int rbc = rb < rowblocks ? rb : rowblocks - 1;
    const int wrow = rbc * 16 + l16;
    const int base = (wrow < m ? wrow : m - 1) * wq;
#pragma unroll
    for (int i = 0; i < KW; ++i)
#pragma unroll
      for (int v = 0; v < 2; ++v) {
        const int g = 2 * l4 + v;
        raw[i][v] = Wp4[base + i * plane + (g < wq ? g : 0)];
      }
    // lane l < 16 KW: coefficient l % KW of row rb * 16 + l / KW; lane l < 16: bias of row rb * 16 + l
    const int ci = rbc * 16 * KW + (lane < 16 * KW ? lane : 0);
    coef = alpha[ci < m * KW ? ci : m * KW - 1];
    const int bi = rbc * 16 + l16;
    bs = a.bias0 ? a.bias0[bi < m ? bi : m - 1] : 0.0f;
  };
  uint4 anext[KW][2];
  float coef_next, bias_next;
  request_rowblock(rb_first + wv, anext, coef_next, bias_next);

  for (int rb = rb_first + wv; rb < rb_end; rb += kWaves) {
    // ---- weight side of the row block, shared by all tiles
    const int wrow_a = rb * 16 + l16;
    const bool wok = wrow_a < m;
    uint4 araw[KW][2];
#pragma unroll
    for (int i = 0; i < KW; ++i)
#pragma unroll
      for (int v = 0; v < 2; ++v)
        araw[i][v] = (wok && 2 * l4 + v < wq) ? anext[i][v] : make_uint4(0, 0, 0, 0);
    const float coef_req = coef_next, bias_req = bias_next;
    request_rowblock(rb + kWaves, anext, coef_next, bias_next);
    // C view: rows 4 * l4 + r
    int crow0 = rb * 16 + 4 * l4;
    bool cok[4];
    float alr[4][KW], bias[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      cok[r] = crow0 + r < m;
#pragma unroll
      for (int i = 0; i < KW; ++i) alr[r][i] = __shfl(coef_req, (4 * l4 + r) * KW + i, kWave);
      bias[r] = __shfl(bias_req, 4 * l4 + r, kWave);
    }
    // ---- contraction with all tiles
    v4f acc[NBT][KW][KA];
    contract_tiles<KW, KA, NBT, true>(araw, tile, acc);

    // ---- epilogue per tile, lane = (batch column l16, row quad l4): the accumulators are the dot products
    // d_ij of the codes (integers, exact in binary32);  y = sum_i alpha_i sum_j beta_j d_ij
#pragma unroll
    for (int bt = 0; bt < NBT; ++bt) {
      float yv[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float y = 0.0f;
#pragma unroll
        for (int i = 0; i < KW; ++i) {
          float inner = 0.0f;
#pragma unroll
          for (int j = 0; j < KA; ++j) inner = fmaf(btv[bt][j], acc[bt][i][j][r], inner);
          y = fmaf(alr[r][i], inner, y);
        }
        yv[r] = y + bias[r];
      }
      if (a.tgt_out && bok[bt]) {  // (no accumulation in this use)
        const long long d = tg[bt] - crow0;
        if (d >= 0 && d < 4) {
          const float yt = d == 0 ? yv[0] : d == 1 ? yv[1] : d == 2 ? yv[2] : yv[3];
          if (crow0 + d < m) a.tgt_out[bcol[bt]] = yt;
        }
      }
      if (a.Y && bok[bt]) {
        float* yp = a.Y + (long long)bcol[bt] * m + crow0;
        if (a.accumulate) {
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (cok[r]) yv[r] += yp[r];
        }
        if ((m & 3) == 0 && cok[3]) {
          // the four rows of this lane are consecutive in Y[b][.]: one aligned 16-byte store
          *reinterpret_cast<float4*>(yp) = make_float4(yv[0], yv[1], yv[2], yv[3]);
        } else {
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (cok[r]) yp[r] = yv[r];
        }
      }
      if (lse_part) {  // uniform: fold this row block's outputs into the running (max, sum)
        float mx = lse_m[bt];
#pragma unroll
        for (int r = 0; r < 4; ++r) mx = fmaxf(mx, cok[r] ? yv[r] : kLseLow);
        float sm = lse_s[bt] * __expf(lse_m[bt] - mx);
#pragma unroll
        for (int r = 0; r < 4; ++r) sm += cok[r] ? __expf(yv[r] - mx) : 0.0f;
        lse_m[bt] = mx;
        lse_s[bt] = sm;
      }
    }
  }

  if (lse_part) {  // uniform
    // One slot per workgroup and batch column: every wave merges its four row quads (lanes 16
    // apart) and leaves the pair in LDS (the staged activations are no longer needed once all
    // waves are past their contractions); wave 0 merges the eight and writes.  A wave that had
    // no row block contributes the neutral pair.
    float2* xch = reinterpret_cast<float2*>(smem);  // [wave][tile][column]
    __syncthreads();
#pragma unroll
    for (int bt = 0; bt < NBT; ++bt) {
      float mm = lse_m[bt], ss = lse_s[bt];
#pragma unroll
      for (int o = 16; o <= 32; o <<= 1) {
        const float m2 = __shfl_xor(mm, o, kWave), s2 = __shfl_xor(ss, o, kWave);
        lse_merge(mm, ss, m2, s2);
      }
      if (l4 == 0) xch[(wv * NBT + bt) * kTileB + l16] = make_float2(mm, ss);
    }
    __syncthreads();
    if (tid < NBT * kTileB) {
      const int b = bg0 + tid;  // tid = tile * 16 + column
      float mm = kLseLow, ss = 0.0f;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        const float2 p = xch[w * NBT * kTileB + tid];
        lse_merge(mm, ss, p.x, p.y);
      }
      if (b < batch) {
        float* dst = lse_part + ((long long)b * a.lse_slots + blockIdx.x) * 2;
        dst[0] = mm;
        dst[1] = ss;
      }
    }
  }
}

// The recurrent steps (Eq. 6 and the GRU) in the same work split, for batches of 128 and more: a
// wave owns 4 hidden units x all gates (the 16 tile rows are 4 units x 4 gates, so that in the C
// layout one lane holds every gate of one unit for one batch entry) x NBT batch tiles x both operand
// blocks, one block after the other, and applies the cell in registers.  Both blocks' activation
// tiles are staged in LDS.  The pre-activations are formed from the exact integer dot products
// (h_t goes back into the on-line quantizer, where a difference in the last digits can move an
// entry across an interval boundary), in the same order as the one-tile kernel.
template <int KW, int KA, int NBT, int EPI, int NWV>
__global__ __launch_bounds__(64 * NWV) void mfma4wc_kernel(BmvArgs a, int rb_per_wg, int rowblocks) {
  static_assert(EPI == kEpiLstm || EPI == kEpiGru, "cell modes only");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int NG = (EPI == kEpiGru) ? 3 : 4;
  constexpr int kGroupB = NBT * kTileB;
  constexpr int kBlockBytes = NBT * KA * kPlaneBytes;
  constexpr int kIter = (NBT * KA * kTileB * 8 + 64 * NWV - 1) / (64 * NWV);
  unsigned char* btile = smem;                                        // [block][tile][plane][kPlaneBytes]
  int* pops = reinterpret_cast<int*>(smem + 2 * kBlockBytes);         // [block][tile][plane][kTileB]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15, l4 = lane >> 4;
  const int bg0 = blockIdx.y * kGroupB;
  const int batch = a.batch;
  const int m = (int)a.m, H = (int)a.H;
  int nlen[2], wq[2];
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    nlen[k] = a.blk[k].n;
    wq[k] = (nlen[k] + 127) >> 7;
  }
  const int rb_first = blockIdx.x * rb_per_wg;
  int rb_end = rb_first + rb_per_wg;
  if (rb_end > rowblocks) rb_end = rowblocks;

  {
    uint4 xw[2][kIter];
#pragma unroll
    for (int k = 0; k < 2; ++k) load_activation_words<KA, NBT, 64 * NWV>(a.blk[k].Xp, batch, bg0, wq[k], xw[k]);
#pragma unroll
    for (int k = 0; k < 2; ++k)
      stage_activation_words<KA, NBT, 64 * NWV>(xw[k], btile + k * kBlockBytes, pops + k * NBT * KA * kTileB);
    __syncthreads();
  }

  // per batch column of this lane (one per tile) and operand block: beta_j and n - 2 popc(x_j)
  int bcol[NBT];
  bool bok[NBT];
  float btv[2][NBT][KA], cx[2][NBT][KA];
#pragma unroll
  for (int bt = 0; bt < NBT; ++bt) {
    bcol[bt] = bg0 + bt * kTileB + l16;
    bok[bt] = bcol[bt] < batch;
    const int bc = bok[bt] ? bcol[bt] : batch - 1;
#pragma unroll
    for (int k = 0; k < 2; ++k)
#pragma unroll
      for (int j = 0; j < KA; ++j) {
        btv[k][bt][j] = a.blk[k].beta[bc * KA + j];
        cx[k][bt][j] = (float)(nlen[k] - 2 * pops[((k * NBT + bt) * KA + j) * kTileB + l16]);
      }
  }

  for (int rb = rb_first + wv; rb < rb_end; rb += NWV) {
    // C view: this lane's hidden unit, rows r = gate r
    const int unit_c = rb * 4 + l4;
    const bool uok = unit_c < H;
    int crow[4];
    float bias0[4], bias1[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      crow[r] = (uok && r < NG) ? r * H + unit_c : 0;
      bias0[r] = a.bias0 ? a.bias0[crow[r]] : 0.0f;
      bias1[r] = (EPI == kEpiGru && a.bias1) ? a.bias1[crow[r]] : 0.0f;
    }
    float prev[NBT];
#pragma unroll
    for (int bt = 0; bt < NBT; ++bt) {
      const int bc = bok[bt] ? bcol[bt] : batch - 1;
      const int t = bc * H + (uok ? unit_c : 0);
      prev[bt] = (EPI == kEpiLstm) ? a.c_prev[t] : a.h_prev[t];
    }
    // A view: lane = (tile row l16 = 4 * unit + gate, k-block l4)
    const int unit_a = rb * 4 + (l16 >> 2), gate_a = l16 & 3;
    const bool wok = unit_a < H && gate_a < NG;
    const int wrow = wok ? gate_a * H + unit_a : 0;

    float ysum[2][NBT][4];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const uint4* Wp4 = reinterpret_cast<const uint4*>(a.blk[k].Wp);
      uint4 araw[KW][2];
      {
        const int base = wrow * wq[k];
        const int plane = m * wq[k];
#pragma unroll
        for (int i = 0; i < KW; ++i)
#pragma unroll
          for (int v = 0; v < 2; ++v) {
            const int g = 2 * l4 + v;
            const uint4 t4 = Wp4[base + i * plane + (g < wq[k] ? g : 0)];
            araw[i][v] = (wok && g < wq[k]) ? t4 : make_uint4(0, 0, 0, 0);
          }
      }
      float alr[4][KW];
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int i = 0; i < KW; ++i) alr[r][i] = a.blk[k].alpha[crow[r] * KW + i];
      // 2 popc of every weight row plane, fetched for the rows of the C view
      float pw2[KW][4];
#pragma unroll
      for (int i = 0; i < KW; ++i) {
        int pc = 0;
#pragma unroll
        for (int v = 0; v < 2; ++v)
          pc += __popc(araw[i][v].x) + __popc(araw[i][v].y) + __popc(araw[i][v].z) + __popc(araw[i][v].w);
        pc += __shfl_xor(pc, 16, kWave);
        pc += __shfl_xor(pc, 32, kWave);
#pragma unroll
        for (int r = 0; r < 4; ++r) pw2[i][r] = (float)(2 * __shfl(pc, 4 * l4 + r, kWave));
      }
      v4f acc[NBT][KW][KA];
      contract_tiles<KW, KA, NBT>(araw, btile + k * kBlockBytes + l16 * 64 + l4 * 16, acc);
      // d_ij = 4 acc_ij - 2 popc(w_i) + (n - 2 popc(x_j)) (integers below 2^24: exact in binary32),
      // y = sum_i alpha_i sum_j beta_j d_ij
#pragma unroll
      for (int bt = 0; bt < NBT; ++bt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          float y = 0.0f;
#pragma unroll
          for (int i = 0; i < KW; ++i) {
            float inner = 0.0f;
#pragma unroll
            for (int j = 0; j < KA; ++j)
              inner = fmaf(btv[k][bt][j], 4.0f * acc[bt][i][j][r] - pw2[i][r] + cx[k][bt][j], inner);
            y = fmaf(alr[r][i], inner, y);
          }
          ysum[k][bt][r] = y;
        }
    }

    // (no early exit for padded batch columns or units: every lane stays active through the
    // loop, the stores are predicated instead)
#pragma unroll
    for (int bt = 0; bt < NBT; ++bt) {
      const int t = bcol[bt] * H + unit_c;
      if constexpr (EPI == kEpiLstm) {
        const float gi = sigmoidf_dev(ysum[0][bt][0] + ysum[1][bt][0] + bias0[0]);
        const float gf = sigmoidf_dev(ysum[0][bt][1] + ysum[1][bt][1] + bias0[1]);
        const float go = sigmoidf_dev(ysum[0][bt][2] + ysum[1][bt][2] + bias0[2]);
        const float gg = tanhf_dev(ysum[0][bt][3] + ysum[1][bt][3] + bias0[3]);
        const float c = fmaf(gf, prev[bt], gi * gg);
        const float h = go * tanhf_dev(c);
        if (bok[bt] && uok) {
          a.c_out[t] = c;
          a.h_out[t] = h;
          if (a.hs_out) a.hs_out[t] = h;
        }
      } else {
        const float rg = sigmoidf_dev(ysum[0][bt][0] + ysum[1][bt][0] + bias0[0] + bias1[0]);
        const float z = sigmoidf_dev(ysum[0][bt][1] + ysum[1][bt][1] + bias0[1] + bias1[1]);
        const float nn = tanhf_dev(fmaf(rg, ysum[1][bt][2] + bias1[2], ysum[0][bt][2] + bias0[2]));
        if (bok[bt] && uok) a.h_out[t] = fmaf(z, prev[bt] - nn, nn);
      }
    }
  }
}

// The recurrent steps when there are too few row-block x batch-tile tasks to give every SIMD more than
// one wave: one workgroup of pair_body per (row-block group, batch group).
template <int KW, int KA, int NBT, int EPI, int NWV>
__global__ __launch_bounds__(64 * NWV) void mfma4p_kernel(BmvArgs a, int rowblocks) {
  __shared__ float4 xch[(NWV / 2) * NBT * 64];  // [pair][tile][lane]: the h-side sums on their way to the x wave
  extern __shared__ __attribute__((aligned(16))) uint4 turn[];
  asm volatile("" ::AMQ_ARG(a.blk[0].Wp), AMQ_ARG(a.blk[0].alpha), AMQ_ARG(a.blk[0].Xp), AMQ_ARG(a.blk[0].beta),
               AMQ_ARG(a.blk[0].n), AMQ_ARG(a.blk[1].Wp), AMQ_ARG(a.blk[1].alpha), AMQ_ARG(a.blk[1].Xp),
               AMQ_ARG(a.blk[1].beta), AMQ_ARG(a.blk[1].n), AMQ_ARG(a.m), AMQ_ARG(a.H), AMQ_ARG(a.batch), AMQ_ARG(a.bias0),
               AMQ_ARG(a.bias1), AMQ_ARG(a.c_prev), AMQ_ARG(a.h_prev), AMQ_ARG(a.h_out), AMQ_ARG(a.c_out),
               AMQ_ARG(a.hs_out), AMQ_ARG(rowblocks));
  pair_body<KW, KA, NBT, EPI, NWV>(a, rowblocks, blockIdx.x, blockIdx.y, turn, xch);
}

// Tiles per wave: as many as keep the accumulators within about 100 registers.
constexpr int max_tiles(int kw, int ka) { return 24 / (kw * ka) > 4 ? 4 : 24 / (kw * ka); }

template <int KW, int KA, int NBT>
hipError_t launch_one(BmvArgs a, hipStream_t s, int* lse_slots) {
  if constexpr (NBT > max_tiles(KW, KA) || NBT < 2) {
    return hipErrorInvalidValue;
  } else {
    const int rowblocks = (int)((a.m + 15) / 16);
    const int groups = (a.batch + NBT * kTileB - 1) / (NBT * kTileB);
    // about one workgroup per compute unit (registers and the staged activations allow no second
    // one); row blocks per workgroup in multiples of 4, so that its four SIMDs (waves w and w + 4
    // share one) get the same number of passes
    int splits = 256 / groups;
    if (splits < 1) splits = 1;
    int per = (rowblocks + splits - 1) / splits;
    per = (per + 3) / 4 * 4;
    if (per < kWaves) per = kWaves;
    const size_t lds = (size_t)NBT * KA * kPlaneBytes + sizeof(int) * NBT * KA * kTileB;
    static std::atomic<unsigned long long> configured{0};
    {
      hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(&mfma4w_kernel<KW, KA, NBT>), (int)lds, configured);
      if (e != hipSuccess) return e;
    }
    dim3 grid((unsigned)((rowblocks + per - 1) / per), (unsigned)groups);
    const long long slots = grid.x;  // one per workgroup of a batch group
    if (slots > kLseMaxSlots || slots > a.lse_cap) a.lse_part = nullptr;
    a.lse_slots = (int)slots;
    if (lse_slots) *lse_slots = a.lse_part ? (int)slots : 0;
    hipLaunchKernelGGL((mfma4w_kernel<KW, KA, NBT>), grid, dim3(64 * kWaves), lds, s, a, per, rowblocks);
    return hipGetLastError();
  }
}

template <int KW, int KA>
hipError_t launch_tiles(const BmvArgs& a, int nbt, hipStream_t s, int* lse_slots) {
  switch (nbt) {
    case 2: return launch_one<KW, KA, 2>(a, s, lse_slots);
    case 3: return launch_one<KW, KA, 3>(a, s, lse_slots);
    case 4: return launch_one<KW, KA, 4>(a, s, lse_slots);
  }
  return hipErrorInvalidValue;
}

template <int KW>
hipError_t launch_ka(const BmvArgs& a, int k_a, int nbt, hipStream_t s, int* lse_slots) {
  switch (k_a) {
    case 1: return launch_tiles<KW, 1>(a, nbt, s, lse_slots);
    case 2: return launch_tiles<KW, 2>(a, nbt, s, lse_slots);
    case 3: return launch_tiles<KW, 3>(a, nbt, s, lse_slots);
    case 4: return launch_tiles<KW, 4>(a, nbt, s, lse_slots);
  }
  return hipErrorInvalidValue;
}

// Batch tiles per wave for this product: the register budget's maximum, lowered so that the
// batch groups come out even (5 tiles -> 3 + 2 rather than 4 + 1).
int tiles_per_wave(int k_w, int k_a, int batch) {
  const int cap = max_tiles(k_w, k_a);
  if (cap < 2) return 0;
  const int tiles = (batch + kTileB - 1) / kTileB;
  const int groups = (tiles + cap - 1) / cap;
  const int nbt = (tiles + groups - 1) / groups;
  return nbt < 2 ? 0 : nbt;
}

// Cell modes: tiles per wave bounded by the accumulators (as above) and by the LDS that both
// operand blocks' activation tiles take (2 * NBT * KA * 8 KiB <= 144 KiB).  With at most four
// plane pairs, two tiles per wave in 8-wave workgroups fit 256 registers and keep two waves on
// every SIMD (each hides the other's load latencies: measured faster than four tiles per wave
// with one wave per SIMD); beyond that, 4-wave workgroups with up to 512 registers per wave.
constexpr int max_cell_tiles(int kw, int ka) {
  if (kw * ka <= 4) return 2;
  int c = max_tiles(kw, ka);
  return 9 / ka < c ? 9 / ka : c;
}
constexpr int cell_waves(int kw, int ka) { return kw * ka <= 4 ? 8 : 4; }
int cell_tiles_per_wave(int k_w, int k_a, int batch) {
  const int cap = max_cell_tiles(k_w, k_a);
  if (cap < 2) return 0;
  const int tiles = (batch + kTileB - 1) / kTileB;
  const int groups = (tiles + cap - 1) / cap;
  const int nbt = (tiles + groups - 1) / groups;
  return nbt < 2 ? 0 : nbt;
}

template <int KW, int KA, int NBT, int EPI>
hipError_t launch_cell_one(const BmvArgs& a, hipStream_t s) {
  if constexpr (NBT > max_cell_tiles(KW, KA) || NBT < 2) {
    return hipErrorInvalidValue;
  } else {
    constexpr int NWV = cell_waves(KW, KA);
    const int rowblocks = (int)((a.H + 3) / 4);
    const int groups = (a.batch + NBT * kTileB - 1) / (NBT * kTileB);
    // about one workgroup per compute unit; row blocks per workgroup in multiples of 4, so that
    // its four SIMDs get the same number of passes
    int splits = 256 / groups;
    if (splits < 1) splits = 1;
    int per = (rowblocks + splits - 1) / splits;
    per = (per + 3) / 4 * 4;
    if (per < NWV) per = NWV;
    const size_t lds = (size_t)2 * NBT * KA * kPlaneBytes + sizeof(int) * 2 * NBT * KA * kTileB;
    static std::atomic<unsigned long long> configured{0};
    {
      hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(&mfma4wc_kernel<KW, KA, NBT, EPI, NWV>), (int)lds,
                                        configured);
      if (e != hipSuccess) return e;
    }
    dim3 grid((unsigned)((rowblocks + per - 1) / per), (unsigned)groups);
    hipLaunchKernelGGL((mfma4wc_kernel<KW, KA, NBT, EPI, NWV>), grid, dim3(64 * NWV), lds, s, a, per, rowblocks);
    return hipGetLastError();
  }
}

template <int KW, int KA, int EPI>
hipError_t launch_cell_tiles(const BmvArgs& a, int nbt, hipStream_t s) {
  switch (nbt) {
    case 2: return launch_cell_one<KW, KA, 2, EPI>(a, s);
    case 3: return launch_cell_one<KW, KA, 3, EPI>(a, s);
    case 4: return launch_cell_one<KW, KA, 4, EPI>(a, s);
  }
  return hipErrorInvalidValue;
}

template <int KW, int EPI>
hipError_t launch_cell_ka(const BmvArgs& a, int k_a, int nbt, hipStream_t s) {
  switch (k_a) {
    case 1: return launch_cell_tiles<KW, 1, EPI>(a, nbt, s);
    case 2: return launch_cell_tiles<KW, 2, EPI>(a, nbt, s);
    case 3: return launch_cell_tiles<KW, 3, EPI>(a, nbt, s);
    case 4: return launch_cell_tiles<KW, 4, EPI>(a, nbt, s);
  }
  return hipErrorInvalidValue;
}

template <int EPI>
hipError_t launch_cell_kw(const BmvArgs& a, int k_w, int k_a, int nbt, hipStream_t s) {
  switch (k_w) {
    case 1: return launch_cell_ka<1, EPI>(a, k_a, nbt, s);
    case 2: return launch_cell_ka<2, EPI>(a, k_a, nbt, s);
    case 3: return launch_cell_ka<3, EPI>(a, k_a, nbt, s);
    case 4: return launch_cell_ka<4, EPI>(a, k_a, nbt, s);
  }
  return hipErrorInvalidValue;
}

// Measured on config 3 (256 row blocks x 4 batch tiles, W3/A3), whole step: one tile per wave in
// workgroups of 8 waves 12.4 us; two tiles per wave in workgroups of 4 (one wave per SIMD, weights
// fetched half as often, activation operands shared by two row blocks instead of four) 13.0 us; two
// tiles, 8 waves (half the compute units) 14.3 us.
template <int KW, int KA, int EPI>
hipError_t launch_pair_one(const BmvArgs& a, hipStream_t s) {
  if constexpr (KW > 3 || KW * KA > 9) {
    return hipErrorInvalidValue;
  } else {
    constexpr int NBT = 1, NWV = 8;
    const int rowblocks = (int)((a.H + 3) / 4);
    const int groups = (a.batch + NBT * kTileB - 1) / (NBT * kTileB);
    dim3 grid((unsigned)((rowblocks + NWV / 2 - 1) / (NWV / 2)), (unsigned)groups);
    BmvArgs b = a;
    AMQ_PHASE_ATTACH(b);
    constexpr size_t lds = pair_body_lds<KW, KA, NBT, NWV>();
    static std::atomic<unsigned long long> configured{0};
    {
      hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(&mfma4p_kernel<KW, KA, NBT, EPI, NWV>), (int)lds,
                                        configured);
      if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((mfma4p_kernel<KW, KA, NBT, EPI, NWV>), grid, dim3(64 * NWV), lds, s, b, rowblocks);
    return hipGetLastError();
  }
}

template <int KW, int EPI>
hipError_t launch_pair_ka(const BmvArgs& a, int k_a, hipStream_t s) {
  switch (k_a) {
    case 1: return launch_pair_one<KW, 1, EPI>(a, s);
    case 2: return launch_pair_one<KW, 2, EPI>(a, s);
    case 3: return launch_pair_one<KW, 3, EPI>(a, s);
    case 4: return launch_pair_one<KW, 4, EPI>(a, s);
  }
  return hipErrorInvalidValue;
}

template <int EPI>
hipError_t launch_pair_kw(const BmvArgs& a, int k_w, int k_a, hipStream_t s) {
  switch (k_w) {
    case 1: return launch_pair_ka<1, EPI>(a, k_a, s);
    case 2: return launch_pair_ka<2, EPI>(a, k_a, s);
    case 3: return launch_pair_ka<3, EPI>(a, k_a, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace

// Recurrent steps with vectors of at most 1024 entries, two or more batch tiles, and at most two
// row-block x tile tasks per SIMD of the chip (beyond that the several-tiles cell kernel takes over;
// a single tile stays with the paired form of the one-tile kernel).
bool mfma4_pair_supported(const BmvArgs& a, int k_w, int k_a, int epi) {
  if (epi != kEpiLstm && epi != kEpiGru) return false;
  if (a.blk[0].n > 1024 || a.blk[1].n > 1024) return false;
  if (k_w > 3 || k_w * k_a > 9) return false;
  const long long tiles = (a.batch + kTileB - 1) / kTileB;
  const long long rowblocks = (a.H + 3) / 4;
  if (tiles < 2 || rowblocks * tiles > 2048) return false;
  if (a.m * 8 * k_w >= (1LL << 31)) return false;  // weight offsets in 16-byte units
  if ((long long)a.batch * a.H >= (1LL << 31)) return false;
  return true;
}

hipError_t launch_mfma4_pair(const BmvArgs& a, int k_w, int k_a, int epi, hipStream_t s) {
  if (epi == kEpiLstm) return launch_pair_kw<kEpiLstm>(a, k_w, k_a, s);
  if (epi == kEpiGru) return launch_pair_kw<kEpiGru>(a, k_w, k_a, s);
  return hipErrorInvalidValue;
}

// Plain products (no integer hook) with vectors of at most 1024 entries, at least two batch tiles,
// and enough row-block tasks to give every SIMD of the chip two of them; sizes whose element
// offsets fit 32 bits.
bool mfma4w_supported(const BmvArgs& a, int k_w, int k_a) {
  if (a.D || a.groups > 1 || a.blk[0].n > 1024 || (!a.Y && !(a.tgt && a.tgt_out))) return false;
  const int nbt = tiles_per_wave(k_w, k_a, a.batch);
  if (nbt == 0) return false;
  if (a.batch > 65535 * nbt * kTileB) return false;
  if (a.m * 8 * k_w >= (1LL << 31)) return false;  // weight offsets in 16-byte units
  if ((long long)a.batch * a.m >= (1LL << 31)) return false;
  const long long rowblocks = (a.m + 15) / 16;
  const long long groups = (a.batch + nbt * kTileB - 1) / (nbt * kTileB);
  return rowblocks * groups >= 2048;
}

hipError_t launch_mfma4w(const BmvArgs& a, int k_w, int k_a, hipStream_t s, int* lse_slots) {
  if (lse_slots) *lse_slots = 0;
  const int nbt = tiles_per_wave(k_w, k_a, a.batch);
  switch (k_w) {
    case 1: return launch_ka<1>(a, k_a, nbt, s, lse_slots);
    case 2: return launch_ka<2>(a, k_a, nbt, s, lse_slots);
    case 3: return launch_ka<3>(a, k_a, nbt, s, lse_slots);
    case 4: return launch_ka<4>(a, k_a, nbt, s, lse_slots);
  }
  return hipErrorInvalidValue;
}

// Recurrent steps with vectors of at most 1024 entries, at least 8 batch tiles, and more row-block x
// batch-tile tasks than the paired-wave form of the one-tile kernel is used for.
bool mfma4w_cell_supported(const BmvArgs& a, int k_w, int k_a, int epi) {
  if (epi != kEpiLstm && epi != kEpiGru) return false;
  if (a.blk[0].n > 1024 || a.blk[1].n > 1024) return false;
  const long long tiles = (a.batch + kTileB - 1) / kTileB;
  const long long rowblocks = (a.H + 3) / 4;
  if (tiles < 8 || rowblocks * tiles <= 2048) return false;
  const int nbt = cell_tiles_per_wave(k_w, k_a, a.batch);
  if (nbt == 0) return false;
  if (a.batch > 65535LL * nbt * kTileB) return false;
  if (a.m * 8 * k_w >= (1LL << 31)) return false;  // weight offsets in 16-byte units
  if ((long long)a.batch * a.H >= (1LL << 31)) return false;
  return true;
}

hipError_t launch_mfma4w_cell(const BmvArgs& a, int k_w, int k_a, int epi, hipStream_t s) {
  const int nbt = cell_tiles_per_wave(k_w, k_a, a.batch);
  if (epi == kEpiLstm) return launch_cell_kw<kEpiLstm>(a, k_w, k_a, nbt, s);
  if (epi == kEpiGru) return launch_cell_kw<kEpiGru>(a, k_w, k_a, nbt, s);
  return hipErrorInvalidValue;
}

}  // namespace amq
