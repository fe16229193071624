// Batched binary matrix products on the fp4 matrix cores of gfx950 (Fig. 3 right: the
// concatenated form), for vectors of at most 1024 entries per operand block.
//
// Why fp4: the contraction only ever multiplies codes, and with both operands written as
// {0, 1} every product and every partial sum (< 2^24) is exact in the E2M1 x E2M1 -> fp32
// MFMA.  v_mfma_scale_f32_16x16x128_f8f6f4 in fp4 mode takes 128 entries of K per instruction
// from 16-byte operands and issues every ~19 cycles on this chip, against ~32 cycles for the
// int8 instruction with 64 entries of K (both measured), i.e. 3.3x the rate per entry.  The
// +-1 inner product is recovered from popcounts:
//   sum_l (2a_l - 1)(2x_l - 1) = 4 * sum_l a_l x_l - 2 * popc(a) - 2 * popc(x) + n.
//
// Expansion: bit p of a packed word becomes nibble 0b0010 (= 1.0 in E2M1) or 0.  One word
// yields the four operand dwords (w << 1, w, w >> 1, w >> 2) & 0x22222222: nibble q of dword s
// is bit 4q + s -- a fixed permutation of K applied to both operands.
//
// Work split: a wave owns 16 tile rows x KW planes x 16 batch entries x KA planes (KW * KA
// accumulators of 4 registers).  A workgroup expands the activation tile (16 batch entries, all
// planes, both operand blocks) into LDS once and its waves walk over row blocks, loading each
// row block's packed weight words straight into the operand layout (lane = row l % 16, words
// 8 * (l / 16) .. + 7).  In the cell modes the 16 tile rows are 4 hidden units x 4 gates, so
// that in the 16x16 C layout (lane: column l % 16, rows 4 * (l / 16) + 0..3) one lane holds all
// gates of one unit for one batch entry and the LSTM / GRU cell is applied in registers.
#include <type_traits>

#include "amq_device.h"
#include "amq_launch.h"

namespace amq {

namespace {

template <int KW, int KA, int EPI, int NWV>
__global__ __launch_bounds__(64 * NWV) void mfma4_kernel(BmvArgs a, int rb_per_wg, int rowblocks) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int NBLK = (EPI == kEpiStore) ? 1 : 2;
  constexpr int NG = (EPI == kEpiGru) ? 3 : 4;
  constexpr int kTileBytes = KA * kPlaneBytes;
  constexpr int kItems = KA * kTileB * 8;             // 16-byte groups of packed words per operand block
  constexpr int kIter = (kItems + 64 * NWV - 1) / (64 * NWV);
  unsigned char* btile = smem;
  int* pops = reinterpret_cast<int*>(smem + NBLK * kTileBytes);  // [NBLK][KA][kTileB]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave index, known uniform to the compiler
  const int l16 = lane & 15, l4 = lane >> 4;
  // phase timers of the profiling build: 0 start, 1 loads issued, 9 own part of the tile staged, 2 barrier passed,
  // 3 column coefficients read, 4 row coefficients spread, 10 weight words used, 5 contraction, 6 epilogue, 8 cell
  AMQ_PHASE_B(AMQ_PHASE_OF(a), 0);
  asm volatile("" ::AMQ_ARG(a.blk[0].Wp), AMQ_ARG(a.blk[0].alpha), AMQ_ARG(a.blk[0].Xp), AMQ_ARG(a.blk[0].beta),
               AMQ_ARG(a.blk[0].n), AMQ_ARG(a.blk[NBLK - 1].Wp), AMQ_ARG(a.blk[NBLK - 1].alpha),
               AMQ_ARG(a.blk[NBLK - 1].Xp), AMQ_ARG(a.blk[NBLK - 1].beta), AMQ_ARG(a.blk[NBLK - 1].n), AMQ_ARG(a.m),
               AMQ_ARG(a.H), AMQ_ARG(a.batch), AMQ_ARG(a.bias0), AMQ_ARG(a.bias1), AMQ_ARG(a.c_prev), AMQ_ARG(a.h_prev),
               AMQ_ARG(a.h_out), AMQ_ARG(a.c_out), AMQ_ARG(a.hs_out), AMQ_ARG(a.Y),
               AMQ_ARG(a.accumulate), AMQ_ARG(rb_per_wg), AMQ_ARG(rowblocks));
  const int b0 = blockIdx.y * kTileB;
  const int batch = a.batch;
  const int m = (int)a.m, H = (int)a.H;
  const uint4* Wp4[NBLK];
  const float* alpha[NBLK];
  int nlen[NBLK], wq[NBLK];
#pragma unroll
  for (int k = 0; k < NBLK; ++k) {
    Wp4[k] = reinterpret_cast<const uint4*>(a.blk[k].Wp);
    alpha[k] = a.blk[k].alpha;
    nlen[k] = a.blk[k].n;
    wq[k] = (nlen[k] + 127) >> 7;  // 16-byte groups per row
  }

  const int b = b0 + l16;
  const bool bok = b < batch;
  const int bc = bok ? b : batch - 1;
  const int rb_first = blockIdx.x * rb_per_wg;
  int rb_end = rb_first + rb_per_wg;
  if (rb_end > rowblocks) rb_end = rowblocks;

  // A-operand view of row block rb: lane = (tile row l16, k-block l4)
  auto a_row = [&](int rb, bool& wok) -> int {
    int wrow;
    if constexpr (EPI == kEpiStore) {
      wrow = rb * 16 + l16;
      wok = wrow < m;
    } else {
      const int unit = rb * 4 + (l16 >> 2);
      const int gate = l16 & 3;
      wok = unit < H && gate < NG;
      wrow = gate * H + unit;
    }
    return wok ? wrow : 0;
  };
  // packed weight words of one operand block of a row block, straight into the operand layout
  auto load_a = [&](auto kc, int rb, uint4 (&araw)[KW][2]) {
    constexpr int k = decltype(kc)::value;
    bool wok;
    const int wrow = a_row(rb, wok);
    const int base = wrow * wq[k];
    const int plane = m * wq[k];
#pragma unroll
    for (int i = 0; i < KW; ++i)
#pragma unroll
      for (int v = 0; v < 2; ++v) {
        const int g = 2 * l4 + v;
        const uint4 t4 = Wp4[k][base + i * plane + (g < wq[k] ? g : 0)];
        araw[i][v] = (wok && g < wq[k]) ? t4 : make_uint4(0, 0, 0, 0);
      }
  };
  // C view of row block rb: rows 4 * l4 + r
  auto c_rows = [&](int rb, int (&crow)[4], bool (&cok)[4]) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      if constexpr (EPI == kEpiStore) {
        crow[r] = rb * 16 + 4 * l4 + r;
        cok[r] = crow[r] < m;
      } else {
        const int unit = rb * 4 + l4;
        cok[r] = unit < H && r < NG;
        crow[r] = r * H + unit;
      }
      if (!cok[r]) crow[r] = 0;
    }
  };
  // Row coefficients of the C view: the 16 lanes of a row quad (same l4) need the same 4 * KW values,
  // so lane l16 < 4 * KW requests one of them (one load per wave instead of 4 * KW) and
  // spread_alpha hands them round through the cross-lane network.
  auto request_alpha = [&](auto kc, int rb) -> float {
    constexpr int k = decltype(kc)::value;
    const int r = l16 / KW, i = l16 % KW;
    int row;
    bool ok;
    if constexpr (EPI == kEpiStore) {
      row = rb * 16 + 4 * l4 + r;
      ok = r < 4 && row < m;
    } else {
      const int unit = rb * 4 + l4;
      ok = r < NG && unit < H;
      row = r * H + unit;
    }
    return alpha[k][(ok ? row : 0) * KW + i];
  };
  auto spread_alpha = [&](float mine, float (&alr)[4][KW]) {
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int i = 0; i < KW; ++i) alr[r][i] = __shfl(mine, 16 * l4 + r * KW + i, kWave);
  };
  // biases of the C view rows the same way: lanes l16 = 0..3 request bias0, 4..7 bias1
  auto request_bias = [&](int rb) -> float {
    const float* src = (l16 & 4) ? ((EPI == kEpiGru) ? a.bias1 : nullptr) : a.bias0;
    const int r = l16 & 3;
    int row;
    bool ok;
    if constexpr (EPI == kEpiStore) {
      row = rb * 16 + 4 * l4 + r;
      ok = row < m;
    } else {
      const int unit = rb * 4 + l4;
      ok = r < NG && unit < H;
      row = r * H + unit;
    }
    return (src && l16 < 8) ? src[ok ? row : 0] : 0.0f;
  };
  using K0 = std::integral_constant<int, 0>;
  using K1 = std::integral_constant<int, NBLK - 1>;

  const int iters = (rb_end - rb_first + NWV - 1) / NWV;

  // ---- prologue: packed activation words of every operand block, 16 bytes per thread, coalesced
  uint4 xw[NBLK][kIter];
#pragma unroll
  for (int k = 0; k < NBLK; ++k) {
    const uint4* Xp4 = reinterpret_cast<const uint4*>(a.blk[k].Xp);
#pragma unroll
    for (int it = 0; it < kIter; ++it) {
      const int e = tid + it * 64 * NWV;
      const int q = e & 7, nn = (e >> 3) & (kTileB - 1), j = e >> 7;
      const bool valid = e < kItems && b0 + nn < batch && q < wq[k];
      const int bb = b0 + nn < batch ? b0 + nn : batch - 1;
      const uint4 v = Xp4[((e < kItems ? j : 0) * batch + bb) * wq[k] + (q < wq[k] ? q : 0)];
      xw[k][it] = valid ? v : make_uint4(0, 0, 0, 0);
    }
  }
  // column coefficients: lane (l16, l4) requests beta[column l16][plane min(l4, KA - 1)] of every block
  float beta_req[NBLK];
#pragma unroll
  for (int k = 0; k < NBLK; ++k) beta_req[k] = a.blk[k].beta[bc * KA + (l4 < KA ? l4 : KA - 1)];
  AMQ_PHASE_B(AMQ_PHASE_OF(a), 1);
#pragma unroll
  for (int k = 0; k < NBLK; ++k) {
#pragma unroll
    for (int it = 0; it < kIter; ++it) {
      const int e = tid + it * 64 * NWV;
      const int q = e & 7, nn = (e >> 3) & (kTileB - 1), j = e >> 7;
      const uint4 w4 = xw[k][it];
      // popcount of the row: its 8 groups sit in 8 consecutive lanes
      const int pc = sum8(__popc(w4.x) + __popc(w4.y) + __popc(w4.z) + __popc(w4.w));
      if (e < kItems) {
        if (q == 0) pops[(k * KA + j) * kTileB + nn] = pc;
        // words 4q .. 4q+3 of the row: k-block q >> 1, steps 4 * (q & 1) + 0..3
        uint4* dst = reinterpret_cast<uint4*>(btile + k * kTileBytes + j * kPlaneBytes +
                                              ((4 * (q & 1)) * kTileB + nn) * 64 + (q >> 1) * 16);
        dst[0 * kTileB * 4] = expand4(w4.x);
        dst[1 * kTileB * 4] = expand4(w4.y);
        dst[2 * kTileB * 4] = expand4(w4.z);
        dst[3 * kTileB * 4] = expand4(w4.w);
      }
    }
  }
  AMQ_PHASE_B(AMQ_PHASE_OF(a), 9);
  lds_barrier();
  AMQ_PHASE_B(AMQ_PHASE_OF(a), 2);

  float btv[NBLK][KA];
  float cx[NBLK][KA];  // n - 2 * popc(activation plane): the column-only part of the dot product
#pragma unroll
  for (int k = 0; k < NBLK; ++k)
#pragma unroll
    for (int j = 0; j < KA; ++j) {
      btv[k][j] = __shfl(beta_req[k], 16 * j + l16, kWave);
      cx[k][j] = (float)(nlen[k] - 2 * pops[(k * KA + j) * kTileB + l16]);
    }

  AMQ_PHASE_B(AMQ_PHASE_OF(a), 3);
  float lse_m = kLseLow, lse_s = 0.0f;  // store mode: running (max, sum exp) of this lane's outputs
  float* const lse_part = (EPI == kEpiStore) ? a.lse_part : nullptr;

  // one operand block of one row block: matrix-core contraction and coefficient epilogue -> ys[r]
  auto run_block = [&](auto kc, const uint4 (&araw)[KW][2], const float (&alr)[4][KW], const int (&crow)[4],
                       const bool (&cok)[4], float (&ys)[4]) {
    constexpr int k = decltype(kc)::value;
    // popcount of every weight row plane: this lane's 8 words, then the four k-blocks of the
    // row (lanes 16 apart), then fetched for the rows of the C view
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

    AMQ_PHASE_B(AMQ_PHASE_OF(a), 10);
    v4f acc[KW][KA];
#pragma unroll
    for (int i = 0; i < KW; ++i)
#pragma unroll
      for (int j = 0; j < KA; ++j) acc[i][j] = v4f{0.f, 0.f, 0.f, 0.f};
    const unsigned char* tile = btile + k * kTileBytes + l16 * 64 + l4 * 16;
    uint4 bop[KA], bnx[KA], aop[KW], anx[KW];
#pragma unroll
    for (int j = 0; j < KA; ++j) bop[j] = *reinterpret_cast<const uint4*>(tile + j * kPlaneBytes);
#pragma unroll
    for (int i = 0; i < KW; ++i) aop[i] = expand4(word_of(araw[i], 0));
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int t = 0; t < kSteps; ++t) {
      if (t + 1 < kSteps) {
#pragma unroll
        for (int j = 0; j < KA; ++j)
          bnx[j] = *reinterpret_cast<const uint4*>(tile + j * kPlaneBytes + (t + 1) * kTileB * 64);
#pragma unroll
        for (int i = 0; i < KW; ++i) anx[i] = expand4(word_of(araw[i], t + 1));
      }
#pragma unroll
      for (int i = 0; i < KW; ++i)
#pragma unroll
        for (int j = 0; j < KA; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(as_operand(aop[i]), as_operand(bop[j]), acc[i][j],
                                                                       4, 4, 0, kScaleOne, 0, kScaleOne);
      // issue order inside a step: the LDS reads of the next step first, then every MFMA
      // followed by up to three of the VALU instructions that expand the next step's weights
      __builtin_amdgcn_sched_group_barrier(0x100, KA, 0);
#pragma unroll
      for (int g = 0; g < KW * KA; ++g) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int j = 0; j < KA; ++j) bop[j] = bnx[j];
#pragma unroll
      for (int i = 0; i < KW; ++i) aop[i] = anx[i];
    }
    // An MFMA reads its operands from all 64 lanes, but the compiler treats it as lane-local
    // and would sink it (and the VALU code producing its operands) into the divergent branch
    // that guards the final stores, where lanes of padded batch columns -- which still supply
    // weight rows -- are masked off.  Pin the accumulators here, in uniform control flow.
#pragma unroll
    for (int i = 0; i < KW; ++i)
#pragma unroll
      for (int j = 0; j < KA; ++j) asm volatile("" : "+v"(acc[i][j]));
    AMQ_PHASE_B(AMQ_PHASE_OF(a), 5);
    // block epilogue in the C view: lane = (batch column l16, row quad l4), with
    //   d_ij = 4 acc_ij - 2 popc(w_i) + (n - 2 popc(x_j))   (integers below 2^24: exact in binary32)
    //   y = sum_i alpha_i sum_j beta_j d_ij.
    if constexpr (EPI == kEpiStore) {
      // plain products (logits): the factored form
      //   4 sum_i alpha_i (sum_j beta_j acc_ij) - (sum_i alpha_i 2 popc(w_i)) (sum_j beta_j)
      //     + (sum_i alpha_i) (sum_j beta_j (n - 2 popc(x_j)))
      // halves the arithmetic; its cancellation costs about one decimal digit (error ~1e-6
      // relative), irrelevant for an output that nothing feeds back into the quantizer
      float sb = 0.0f, sbcx = 0.0f;
#pragma unroll
      for (int j = 0; j < KA; ++j) {
        sb += btv[k][j];
        sbcx = fmaf(btv[k][j], cx[k][j], sbcx);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float y = 0.0f, pa = 0.0f, sa = 0.0f;
#pragma unroll
        for (int i = 0; i < KW; ++i) {
          float inner = 0.0f;
#pragma unroll
          for (int j = 0; j < KA; ++j) inner = fmaf(btv[k][j], acc[i][j][r], inner);
          y = fmaf(alr[r][i], inner, y);
          pa = fmaf(alr[r][i], pw2[i][r], pa);
          sa += alr[r][i];
        }
        ys[r] = fmaf(4.0f, y, fmaf(sa, sbcx, -pa * sb));
      }
      if (a.D && bok) {  // integer test hook: the dot products themselves
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (cok[r]) {
#pragma unroll
            for (int i = 0; i < KW; ++i)
#pragma unroll
              for (int j = 0; j < KA; ++j)
                a.D[(((long long)b * m + crow[r]) * KW + i) * KA + j] = (int)(4.0f * acc[i][j][r] - pw2[i][r] + cx[k][j]);
          }
      }
    } else {
      // recurrent cells: h_t goes back into the on-line quantizer, where a difference in the
      // last digits can move an entry across an interval boundary; form the exact integer
      // dot products first, as the reference arithmetic does
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float y = 0.0f;
#pragma unroll
        for (int i = 0; i < KW; ++i) {
          float inner = 0.0f;
#pragma unroll
          for (int j = 0; j < KA; ++j) inner = fmaf(btv[k][j], 4.0f * acc[i][j][r] - pw2[i][r] + cx[k][j], inner);
          y = fmaf(alr[r][i], inner, y);
        }
        ys[r] = y;
      }
    }
  };
  for (int it = 0; it < iters; ++it) {
    const int rb = rb_first + it * NWV + wv;
    if (rb >= rb_end) break;
    float ysum[NBLK][4];
    int crow[4];
    bool cok[4];
    float bias0[4], bias1[4], yold[4], prev = 0.0f;
    {
      c_rows(rb, crow, cok);
      uint4 araw[NBLK][KW][2];
      float alr[NBLK][4][KW];
      load_a(K0{}, rb, araw[0]);
      if constexpr (NBLK == 2) load_a(K1{}, rb, araw[NBLK - 1]);
      const float alpha_req0 = request_alpha(K0{}, rb);
      const float alpha_req1 = (NBLK == 2) ? request_alpha(K1{}, rb) : 0.0f;
      const float bias_req = request_bias(rb);
#pragma unroll
      for (int r = 0; r < 4; ++r)
        yold[r] = (EPI == kEpiStore && a.accumulate && a.Y) ? a.Y[(long long)bc * m + crow[r]] : 0.0f;
      if constexpr (EPI == kEpiLstm) prev = a.c_prev[bc * H + crow[0]];
      if constexpr (EPI == kEpiGru) prev = a.h_prev[bc * H + crow[0]];
      spread_alpha(alpha_req0, alr[0]);
      if constexpr (NBLK == 2) spread_alpha(alpha_req1, alr[NBLK - 1]);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        bias0[r] = __shfl(bias_req, 16 * l4 + r, kWave);
        bias1[r] = __shfl(bias_req, 16 * l4 + 4 + r, kWave);
      }
      AMQ_PHASE_B(AMQ_PHASE_OF(a), 4);
      run_block(K0{}, araw[0], alr[0], crow, cok, ysum[0]);
      if constexpr (NBLK == 2) run_block(K1{}, araw[NBLK - 1], alr[NBLK - 1], crow, cok, ysum[NBLK - 1]);
    }
    AMQ_PHASE_B(AMQ_PHASE_OF(a), 6);

    // (no early exit for padded batch columns: every lane stays active through the loop, the
    // stores below are predicated instead)
    if constexpr (EPI == kEpiStore) {
      float yv[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) yv[r] = ysum[0][r] + bias0[r] + yold[r];
      if (a.Y && bok) {
        float* yp = a.Y + (long long)b * m + crow[0];
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
        float mx = lse_m;
#pragma unroll
        for (int r = 0; r < 4; ++r) mx = fmaxf(mx, cok[r] ? yv[r] : kLseLow);
        float sm = lse_s * __expf(lse_m - mx);
#pragma unroll
        for (int r = 0; r < 4; ++r) sm += cok[r] ? __expf(yv[r] - mx) : 0.0f;
        lse_m = mx;
        lse_s = sm;
      }
    } else if constexpr (EPI == kEpiLstm) {
      if (bok && cok[0]) {
        const int t = b * H + crow[0];
        const float gi = sigmoidf_dev(ysum[0][0] + ysum[1][0] + bias0[0]);
        const float gf = sigmoidf_dev(ysum[0][1] + ysum[1][1] + bias0[1]);
        const float go = sigmoidf_dev(ysum[0][2] + ysum[1][2] + bias0[2]);
        const float gg = tanhf_dev(ysum[0][3] + ysum[1][3] + bias0[3]);
        const float c = fmaf(gf, prev, gi * gg);
        const float h = go * tanhf_dev(c);
        a.c_out[t] = c;
        a.h_out[t] = h;
        if (a.hs_out) a.hs_out[t] = h;
      }
      AMQ_PHASE_B(AMQ_PHASE_OF(a), 8 + 8 * it);
    } else {
      if (bok && cok[0]) {
        const int t = b * H + crow[0];
        const float rg = sigmoidf_dev(ysum[0][0] + ysum[1][0] + bias0[0] + bias1[0]);
        const float z = sigmoidf_dev(ysum[0][1] + ysum[1][1] + bias0[1] + bias1[1]);
        const float nn = tanhf_dev(fmaf(rg, ysum[1][2] + bias1[2], ysum[0][2] + bias0[2]));
        a.h_out[t] = fmaf(z, prev - nn, nn);
      }
    }
  }
  if constexpr (EPI == kEpiStore) {
    if (lse_part) {
      // one slot per wave and batch column: merge the four row quads (lanes 16 apart); a wave
      // that had no row block writes the neutral pair
#pragma unroll
      for (int o = 16; o <= 32; o <<= 1) {
        const float m2 = __shfl_xor(lse_m, o, kWave), s2 = __shfl_xor(lse_s, o, kWave);
        lse_merge(lse_m, lse_s, m2, s2);
      }
      if (l4 == 0 && bok) {
        float* dst = lse_part + ((long long)b * a.lse_slots + blockIdx.x * NWV + wv) * 2;
        dst[0] = lse_m;
        dst[1] = lse_s;
      }
    }
  }
}

template <int KW, int KA, int EPI, int NWV>
hipError_t launch_one(BmvArgs a, int rowblocks, int rb_per_wg, hipStream_t s, int* lse_slots) {
  constexpr int NBLK = (EPI == kEpiStore) ? 1 : 2;
  // activation tiles and their popcounts (padded to 16 bytes)
  const size_t lds = (size_t)NBLK * KA * kSteps * kTileB * 64 + 16 * ((sizeof(int) * NBLK * KA * kTileB + 15) / 16);
  static std::atomic<unsigned long long> configured{0};
  {
    hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(&mfma4_kernel<KW, KA, EPI, NWV>), (int)lds, configured);
    if (e != hipSuccess) return e;
  }
  AMQ_PHASE_ATTACH(a);
  dim3 grid((unsigned)((rowblocks + rb_per_wg - 1) / rb_per_wg), (unsigned)((a.batch + kTileB - 1) / kTileB));
  const long long slots = (long long)grid.x * NWV;  // one per wave of a batch tile's workgroups
  if (EPI != kEpiStore || slots > kLseMaxSlots || slots > a.lse_cap) a.lse_part = nullptr;
  a.lse_slots = (int)slots;
  if (lse_slots) *lse_slots = a.lse_part ? (int)slots : 0;
  hipLaunchKernelGGL((mfma4_kernel<KW, KA, EPI, NWV>), grid, dim3(64 * NWV), lds, s, a, rb_per_wg, rowblocks);
  return hipGetLastError();
}

template <int KW, int KA, int EPI>
hipError_t launch_mode(const BmvArgs& a, hipStream_t s, int* lse_slots) {
  const int rowblocks = (int)((EPI == kEpiStore) ? (a.m + 15) / 16 : (a.H + 3) / 4);
  const int btiles = (a.batch + kTileB - 1) / kTileB;
  // about two workgroups per CU; each expands its activation tile once and then walks row blocks
  int splits = (512 + btiles - 1) / btiles;
  int per = (rowblocks + splits - 1) / splits;
  if (per < 4) per = 4;
  // 8 waves (two per SIMD) when there is work for them and 256 registers per wave suffice
  if constexpr (KW * KA <= (EPI == kEpiStore ? 9 : 4))
    if (per >= 16) return launch_one<KW, KA, EPI, 8>(a, rowblocks, per, s, lse_slots);
  return launch_one<KW, KA, EPI, 4>(a, rowblocks, per, s, lse_slots);
}

template <int KW, int KA>
hipError_t launch_epi(const BmvArgs& a, int epi, hipStream_t s, int* lse_slots) {
  switch (epi) {
    case kEpiStore: return launch_mode<KW, KA, kEpiStore>(a, s, lse_slots);
    case kEpiLstm: return launch_mode<KW, KA, kEpiLstm>(a, s, lse_slots);
    case kEpiGru: return launch_mode<KW, KA, kEpiGru>(a, s, lse_slots);
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

// Vectors of at most 1024 entries, and sizes whose element offsets fit 32 bits.
bool mfma4_supported(const BmvArgs& a, int k_w, int epi) {
  const int nblk = (epi == kEpiStore) ? 1 : 2;
  for (int k = 0; k < nblk; ++k)
    if (a.blk[k].n > 1024) return false;
  if (a.batch > 65535 * kTileB) return false;
  if (a.m * 8 * k_w >= (1LL << 31)) return false;       // weight offsets in 16-byte units
  if ((long long)a.batch * (a.m > a.H ? a.m : a.H) >= (1LL << 31)) return false;
  return true;
}

hipError_t launch_mfma4(BmvArgs a, int k_w, int k_a, int epi, hipStream_t s, int* lse_slots) {
  if (lse_slots) *lse_slots = 0;
  if (epi != kEpiStore) a.lse_part = nullptr;
  switch (k_w) {
    case 1: return launch_ka<1>(a, k_a, epi, s, lse_slots);
    case 2: return launch_ka<2>(a, k_a, epi, s, lse_slots);
    case 3: return launch_ka<3>(a, k_a, epi, s, lse_slots);
    case 4: return launch_ka<4>(a, k_a, epi, s, lse_slots);
  }
  return hipErrorInvalidValue;
}

}  // namespace amq
