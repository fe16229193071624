// Body of the recurrent-step product kernel for few row-block x batch-tile tasks (config 3's batch of
// 64: 256 row blocks x 4 tiles): products with both weight blocks on the fp4 matrix cores, coefficient
// epilogue and cell (Eq. 6 and Sec. 4, Fig. 3 right), for one workgroup.
//
// Such a launch is bound by what one wave issues from start to end, so this form cuts the per-wave path:
//   * a wave takes ONE operand block (the x block and the h block of a row block go to two paired
//     waves; the h-side sums cross through LDS) and NBT batch tiles per set of weight words;
//   * every request is contiguous (8 adjacent lanes take one 128-byte row).  In the operand layout
//     adjacent lanes are adjacent rows, 128 bytes apart, and a compute unit needs three times as long
//     to serve such loads (measured for 12 KiB per wave: complete after 3.3 K / 6.2 K cycles for the
//     first / second wave of a SIMD, against 1.7 K / 2.7 K cycles for contiguous ones);
//   * operands are {-1, +1} codes (expand4_signed), so the accumulators hold the inner products of the
//     codes themselves: no popcounts.  Positions past the end of a vector are 0 bits in both operands,
//     i.e. (-1)(-1) = +1 each, a constant that the epilogue takes off.  On this chip the fp4 matrix
//     instruction and vector instructions do not overlap, neither within a wave nor between the two
//     waves of a SIMD (measured: 17 cycles per matrix instruction plus 4 per vector instruction,
//     strictly additive), so the expansion work is what there is to save:
//   * the activation operands of the batch tile (both operand blocks) are expanded once per workgroup:
//     each wave fetches its share of the packed words, expands them and writes them to LDS where the
//     matrix instruction wants them; one barrier, then every wave reads its operands per k-step;
//   * the weight words of a wave's 16 rows are turned into the operand layout through a private piece
//     of LDS (one plane at a time, rows padded to 144 bytes, no barrier: LDS serves one wave's accesses
//     in order) and expanded in registers, one k-step ahead.  Lane (row, k-block b) holds the 16-byte
//     pieces b and b + 4 of its row -- which K positions a k-block holds is free as long as both
//     operands agree.
// Workgroups of NWV waves (NWV / 2 row blocks x 2 operand blocks).  Same arithmetic and summation
// order as the other cell kernels: results are bit-identical to theirs.
//
// The step can also be cut in two along the operand blocks (Eq. 6: W_x x_t does not depend on the
// recurrence): kPairXOnly forms the x-side sums of NWV row blocks and stores them, kPairHOnly forms the
// h-side sums, adds the stored x-side sums in the order the whole step adds them, and applies the cell.
// The stored sums are exactly the values that otherwise travel from the x wave's registers, so the
// results stay bit-identical.
#pragma once
#include "amq_device.h"
#include "amq_launch.h"

namespace amq {

constexpr int kTurnStride = 9;  // 16-byte units per row in the LDS piece that turns rows into operands (128 B + 16 B pad)

// Which part of the step a workgroup forms.  The x-side sums of the split form live in a.Y as
// [batch][hidden unit][4 gates] binary32 (16 bytes per (entry, unit): one store / load per lane).
enum { kPairBoth = 0, kPairXOnly = 1, kPairHOnly = 2 };

// Dynamic LDS of the body: activation operand images [block][tile][plane][k-step][64 lanes] x 16 B, then
// one padded 16-row tile per wave.
template <int KW, int KA, int NBT, int NWV, int MODE = kPairBoth>
constexpr size_t pair_body_lds() {
  return sizeof(uint4) * ((MODE == kPairBoth ? 2 : 1) * NBT * KA * kSteps * 64 + NWV * kTileB * kTurnStride);
}
// Row blocks (of 4 hidden units) per workgroup.
template <int NWV, int MODE>
constexpr int pair_body_rowblocks() {
  return MODE == kPairBoth ? NWV / 2 : NWV;
}

// bx, by: row-block group and batch group of this workgroup.  turn: pair_body_lds() bytes of LDS, 16-byte
// aligned.  xch (kPairBoth only): (NWV / 2) * NBT * 64 float4 of LDS.
template <int KW, int KA, int NBT, int EPI, int NWV, int MODE = kPairBoth>
__device__ __forceinline__ void pair_body(const BmvArgs& a, int rowblocks, int bx, int by, uint4* turn, float4* xch) {
  static_assert(EPI == kEpiLstm || EPI == kEpiGru, "cell modes only");
  constexpr int NG = (EPI == kEpiGru) ? 3 : 4;
  constexpr int NBLK = MODE == kPairBoth ? 2 : 1;  // operand blocks whose activations the workgroup stages

  // (phase timers of the profiling build: 0 start, 1 first requests issued, 9 activation operands written,
  // 2 barrier, 4 weight words in operand layout, 10 first operands expanded, 5 contraction, 6 epilogue,
  // 7 exchange, 8 cell)
  AMQ_PHASE_WHEN(bx == 0 && by == 0, AMQ_PHASE_OF(a), 8, 0);
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15, l4 = lane >> 4;
  // row block of the workgroup, operand block (0: x, 1: h; in the whole step the x wave applies the cell)
  const int pr = MODE == kPairBoth ? wv >> 1 : wv;
  const int kb = MODE == kPairBoth ? (wv & 1) : MODE == kPairHOnly ? 1 : 0;
  constexpr bool kCellHere = MODE != kPairXOnly;  // this workgroup applies the cell (its kb == 0 waves in kPairBoth)
  const int bg0 = by * NBT * kTileB;
  const int batch = a.batch;
  const int m = (int)a.m, H = (int)a.H;
  const int rb = bx * pair_body_rowblocks<NWV, MODE>() + pr;
  const bool live = rb < rowblocks;  // (a wave without a row block still meets the barriers)

  const float* alpha = kb ? a.blk[1].alpha : a.blk[0].alpha;
  const float* beta = kb ? a.blk[1].beta : a.blk[0].beta;
  const int nlen = kb ? a.blk[1].n : a.blk[0].n;
  const int wq = (nlen + 127) >> 7;  // 16-byte pieces per row
  const int ld_piece = lane & 7;

  // ---- requests.  All are a uniform base plus a 32-bit byte offset per lane, in straight-line code (with
  // loads in conditional blocks the compiler waits for all of them before the first use of any).  Rows,
  // gates and columns past the end are clamped to the last valid one (their results are never stored);
  // pieces past the end of a short row are fetched from piece 0 and masked to zero bits.
  //
  // Activation words, shared by the workgroup: both operand blocks' tiles are kShareReq requests of 1 KiB
  // (block, tile, plane, half: batch columns 8v .. 8v + 7 of the tile, lane -> column lane / 8, piece
  // lane % 8); wave w issues requests w, w + NWV, ...  A wave whose share is one request short repeats
  // the last one: same bytes to the same place.
  constexpr int kShareReq = NBLK * NBT * KA * 2;
  constexpr int kSharePer = (kShareReq + NWV - 1) / NWV;
  uint4 bshare[kSharePer];
  uint32_t bshare_keep[kSharePer];  // all ones, or zero for a lane past the end of a short row
  auto request_activations = [&]() {
#pragma unroll
    for (int q = 0; q < kSharePer; ++q) {
      int idx = wv + q * NWV;  // (uniform)
      idx = idx < kShareReq ? idx : kShareReq - 1;
      const int v = idx & 1, j = (idx >> 1) % KA, bt = (idx >> 1) / KA % NBT;
      const int k2 = MODE == kPairBoth ? idx / (2 * KA * NBT) : kb;
      const int n2 = k2 ? a.blk[1].n : a.blk[0].n;
      const int wq2 = (n2 + 127) >> 7;
      const char* Xb = reinterpret_cast<const char*>(k2 ? a.blk[1].Xp : a.blk[0].Xp);
      int col = bg0 + bt * kTileB + 8 * v + (lane >> 3);
      col = col < batch ? col : batch - 1;
      bshare_keep[q] = ld_piece < wq2 ? 0xffffffffu : 0u;
      const unsigned off = (unsigned)(col * wq2 + (ld_piece < wq2 ? ld_piece : 0)) * 16u;
      bshare[q] = *reinterpret_cast<const uint4*>(Xb + (size_t)j * batch * wq2 * 16 + off);
    }
  };
  // Weight words, private to the wave: request v of plane i covers gates 2v and 2v + 1 of the row
  // block's 4 units, 512 contiguous bytes each (lane -> gate 2v + lane / 32, unit (lane / 8) % 4, piece
  // lane % 8).
  uint4 araw[KW][2];
  const uint32_t a_keep = ld_piece < wq ? 0xffffffffu : 0u;
  auto request_weights = [&]() {
    int unit = rb * 4 + ((lane >> 3) & 3);
    unit = unit < H ? unit : H - 1;
    const char* Wb = reinterpret_cast<const char*>(kb ? a.blk[1].Wp : a.blk[0].Wp);
    const size_t wplane = (size_t)m * wq * 16;
#pragma unroll
    for (int v = 0; v < 2; ++v) {
      int gate_row = 2 * v + (lane >> 5);
      gate_row = gate_row < NG ? gate_row : NG - 1;
      const unsigned aoff = (unsigned)((gate_row * H + unit) * wq + (ld_piece < wq ? ld_piece : 0)) * 16u;
#pragma unroll
      for (int i = 0; i < KW; ++i) araw[i][v] = *reinterpret_cast<const uint4*>(Wb + i * wplane + aoff);
    }
  };
  // The small operands of the epilogue: scattered 4-byte loads, each of which holds up the memory pipe
  // far longer than its size suggests, so they are kept away from the operand requests.
  int bcol[NBT];
  bool bok[NBT];
  float beta_req[NBT];
#pragma unroll
  for (int bt = 0; bt < NBT; ++bt) {
    bcol[bt] = bg0 + bt * kTileB + l16;
    bok[bt] = bcol[bt] < batch;
    beta_req[bt] = 0.0f;
  }
  const int unit_c = rb * 4 + l4;
  const bool uok = live && unit_c < H;
  const bool cell_wave = kCellHere && (MODE == kPairHOnly || kb == 0);
  float alpha_req = 0.0f, bias_req = 0.0f, prev[NBT];
  float4 xside[NBT];  // kPairHOnly: the stored x-side sums of this lane's (entry, unit)
#pragma unroll
  for (int bt = 0; bt < NBT; ++bt) {
    prev[bt] = 0.0f;
    xside[bt] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
  auto request_column_coefficients = [&]() {
#pragma unroll
    for (int bt = 0; bt < NBT; ++bt) {
      const int bc = bok[bt] ? bcol[bt] : batch - 1;
      // lane (l16, l4) asks for plane min(l4, KA - 1) of its column
      beta_req[bt] = beta[bc * KA + (l4 < KA ? l4 : KA - 1)];
    }
  };
  auto request_row_operands = [&]() {
    // row coefficients (lane l16 < 4 * KW asks for one of the 4 * KW values its row quad needs), and for
    // the wave that applies the cell the biases and the previous state
    const int r = l16 / KW, i = l16 % KW;
    alpha_req = alpha[((uok && r < NG) ? r * H + unit_c : 0) * KW + i];
    if (cell_wave) {
      const float* src = (l16 & 4) ? ((EPI == kEpiGru) ? a.bias1 : nullptr) : a.bias0;
      const int rr = l16 & 3;
      bias_req = (src && l16 < 8) ? src[(uok && rr < NG) ? rr * H + unit_c : 0] : 0.0f;
#pragma unroll
      for (int bt = 0; bt < NBT; ++bt) {
        const int t = (bok[bt] ? bcol[bt] : batch - 1) * H + (uok ? unit_c : 0);
        prev[bt] = (EPI == kEpiLstm) ? a.c_prev[t] : a.h_prev[t];
        if constexpr (MODE == kPairHOnly) xside[bt] = reinterpret_cast<const float4*>(a.Y)[t];
      }
    }
  };

  uint4* const image = turn;  // [block][tile][plane][k-step][64]
  uint4* const mine = turn + kShareReq / 2 * kSteps * 64 + wv * (kTileB * kTurnStride);
  // Weights: rows -> operand layout through this wave's private piece of LDS, plane after plane; tile row
  // l16 = 4 * unit + gate, lane (l16, l4) takes pieces l4 and l4 + 4.
  auto turn_weights = [&]() {
    const int row = 4 * ((lane >> 3) & 3) + (lane >> 5);
#pragma unroll
    for (int i = 0; i < KW; ++i) {
#pragma unroll
      for (int v = 0; v < 2; ++v)
        mine[(row + 2 * v) * kTurnStride + ld_piece] =
            make_uint4(araw[i][v].x & a_keep, araw[i][v].y & a_keep, araw[i][v].z & a_keep, araw[i][v].w & a_keep);
#pragma unroll
      for (int v = 0; v < 2; ++v) araw[i][v] = mine[l16 * kTurnStride + l4 + 4 * v];
    }
  };
  // Activations: the lane that fetched piece p of batch column c expands its four words to {-1, +1}
  // codes and puts each where the matrix instruction wants it: the image of (block, tile, plane, k-step
  // t) is 64 lanes x 16 bytes, and lane (column c, k-block b) of step t uses word t % 4 of piece b +
  // 4 * (t / 4).  The column index is xor-ed with a value that depends on (b, t / 4), which makes both
  // these writes and the reads of the contraction conflict-free.
  auto expand_activations = [&]() {
    const int c = lane >> 3, pb = ld_piece & 3, th = ld_piece >> 2;
    const int swz = (pb << 1) | (th << 3);
#pragma unroll
    for (int q = 0; q < kSharePer; ++q) {
      int idx = wv + q * NWV;
      idx = idx < kShareReq ? idx : kShareReq - 1;
      uint4* dst = image + ((idx >> 1) * kSteps + 4 * th) * 64 + 16 * pb + ((8 * (idx & 1) + c) ^ swz);
      dst[0 * 64] = expand4_signed(bshare[q].x & bshare_keep[q]);
      dst[1 * 64] = expand4_signed(bshare[q].y & bshare_keep[q]);
      dst[2 * 64] = expand4_signed(bshare[q].z & bshare_keep[q]);
      dst[3 * 64] = expand4_signed(bshare[q].w & bshare_keep[q]);
    }
  };

  request_activations();
  __builtin_amdgcn_sched_barrier(0);  // the shared requests go out first: every wave waits for them
  request_weights();
  AMQ_PHASE_WHEN(bx == 0 && by == 0, AMQ_PHASE_OF(a), 8, 1);
  expand_activations();
  AMQ_PHASE_WHEN(bx == 0 && by == 0, AMQ_PHASE_OF(a), 8, 9);
  lds_barrier();
  AMQ_PHASE_WHEN(bx == 0 && by == 0, AMQ_PHASE_OF(a), 8, 2);
  turn_weights();
  AMQ_PHASE_WHEN(bx == 0 && by == 0, AMQ_PHASE_OF(a), 8, 4);
  // this lane's operand of (tile, plane, k-step)
  const uint4* const myimage = image + (MODE == kPairBoth ? kb : 0) * (NBT * KA * kSteps * 64) + 16 * l4;
  auto b_operand = [&](int bt, int j, int t) {
    return myimage[((bt * KA + j) * kSteps + t) * 64 + (l16 ^ ((l4 << 1) | ((t >> 2) << 3)))];
  };

  // ---- contraction: k-step t multiplies the t-th words of this lane's k-block; the operands of step
  // t + 1 are fetched / expanded before the matrix instructions of step t
  v4f acc[NBT][KW][KA];
#pragma unroll
  for (int bt = 0; bt < NBT; ++bt)
#pragma unroll
    for (int i = 0; i < KW; ++i)
#pragma unroll
      for (int j = 0; j < KA; ++j) acc[bt][i][j] = v4f{0.f, 0.f, 0.f, 0.f};
  uint4 aop[KW], anx[KW], bop[NBT][KA], bnx[NBT][KA];
#pragma unroll
  for (int bt = 0; bt < NBT; ++bt)
#pragma unroll
    for (int j = 0; j < KA; ++j) bop[bt][j] = b_operand(bt, j, 0);
#pragma unroll
  for (int i = 0; i < KW; ++i) aop[i] = expand4_signed(word_of(araw[i], 0));
  AMQ_PHASE_WHEN(bx == 0 && by == 0, AMQ_PHASE_OF(a), 8, 10);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int t = 0; t < kSteps; ++t) {
    if (t + 1 < kSteps) {
#pragma unroll
      for (int bt = 0; bt < NBT; ++bt)
#pragma unroll
        for (int j = 0; j < KA; ++j) bnx[bt][j] = b_operand(bt, j, t + 1);
#pragma unroll
      for (int i = 0; i < KW; ++i) anx[i] = expand4_signed(word_of(araw[i], t + 1));
    }
#pragma unroll
    for (int bt = 0; bt < NBT; ++bt)
#pragma unroll
      for (int i = 0; i < KW; ++i)
#pragma unroll
        for (int j = 0; j < KA; ++j)
          acc[bt][i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(as_operand(aop[i]), as_operand(bop[bt][j]),
                                                                           acc[bt][i][j], 4, 4, 0, kScaleOne, 0, kScaleOne);
    __builtin_amdgcn_sched_barrier(0);
    if (t == 0) {
      // under the contraction: here they return before the epilogue and delay no operand request
      request_column_coefficients();
      request_row_operands();
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int i = 0; i < KW; ++i) aop[i] = anx[i];
#pragma unroll
    for (int bt = 0; bt < NBT; ++bt)
#pragma unroll
      for (int j = 0; j < KA; ++j) bop[bt][j] = bnx[bt][j];
  }
  // An MFMA reads its operands from all 64 lanes, but the compiler treats it as lane-local and
  // would sink it into the divergent branches that guard the stores of the epilogue, where lanes of
  // padded batch columns -- which still supply weight rows -- are masked off.  Pin the accumulators
  // here, in uniform control flow.
#pragma unroll
  for (int bt = 0; bt < NBT; ++bt)
#pragma unroll
    for (int i = 0; i < KW; ++i)
#pragma unroll
      for (int j = 0; j < KA; ++j) asm volatile("" : "+v"(acc[bt][i][j]));
  AMQ_PHASE_WHEN(bx == 0 && by == 0, AMQ_PHASE_OF(a), 8, 5);

  // ---- epilogue: d_ij = acc_ij - (1024 - n) are the dot products of the codes (integers, exact in
  // binary32); y = sum_i alpha_i sum_j beta_j d_ij
  float btv[NBT][KA];
#pragma unroll
  for (int bt = 0; bt < NBT; ++bt)
#pragma unroll
    for (int j = 0; j < KA; ++j) btv[bt][j] = __shfl(beta_req[bt], 16 * j + l16, kWave);
  float alr[4][KW];
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int i = 0; i < KW; ++i) alr[r][i] = __shfl(alpha_req, 16 * l4 + r * KW + i, kWave);
  const float pad = (float)(kSteps * 128 - nlen);
  float ysum[NBT][4];
#pragma unroll
  for (int bt = 0; bt < NBT; ++bt)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      float y = 0.0f;
#pragma unroll
      for (int i = 0; i < KW; ++i) {
        float inner = 0.0f;
#pragma unroll
        for (int j = 0; j < KA; ++j) inner = fmaf(btv[bt][j], acc[bt][i][j][r] - pad, inner);
        y = fmaf(alr[r][i], inner, y);
      }
      ysum[bt][r] = y;
    }
  AMQ_PHASE_WHEN(bx == 0 && by == 0, AMQ_PHASE_OF(a), 8, 6);
  if constexpr (MODE == kPairXOnly) {
    // the x-side sums of (entry, unit), all gates, as one 16-byte store
#pragma unroll
    for (int bt = 0; bt < NBT; ++bt)
      if (bok[bt] && uok)
        reinterpret_cast<float4*>(a.Y)[bcol[bt] * H + unit_c] = make_float4(ysum[bt][0], ysum[bt][1], ysum[bt][2], ysum[bt][3]);
    return;
  }
  if constexpr (MODE == kPairBoth) {
    if (kb == 1) {
#pragma unroll
      for (int bt = 0; bt < NBT; ++bt)
        xch[(pr * NBT + bt) * 64 + lane] = make_float4(ysum[bt][0], ysum[bt][1], ysum[bt][2], ysum[bt][3]);
    }
    lds_barrier();
    AMQ_PHASE_WHEN(bx == 0 && by == 0, AMQ_PHASE_OF(a), 8, 7);
    if (kb != 0) return;
  }
  float bias0[4], bias1[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    bias0[r] = __shfl(bias_req, 16 * l4 + r, kWave);
    bias1[r] = __shfl(bias_req, 16 * l4 + 4 + r, kWave);
  }
  // (no early exit for padded batch columns or units: every lane stays active, the stores are predicated)
#pragma unroll
  for (int bt = 0; bt < NBT; ++bt) {
    // x-side and h-side sums of this lane's (entry, unit): in the whole step this wave formed the x side and
    // the h side comes through LDS; in the split step the x side was stored by the earlier launch
    float yx[4], yh[4];
    if constexpr (MODE == kPairBoth) {
      const float4 o = xch[(pr * NBT + bt) * 64 + lane];
      yh[0] = o.x; yh[1] = o.y; yh[2] = o.z; yh[3] = o.w;
#pragma unroll
      for (int r = 0; r < 4; ++r) yx[r] = ysum[bt][r];
    } else {
      yx[0] = xside[bt].x; yx[1] = xside[bt].y; yx[2] = xside[bt].z; yx[3] = xside[bt].w;
#pragma unroll
      for (int r = 0; r < 4; ++r) yh[r] = ysum[bt][r];
    }
    const int t = bcol[bt] * H + unit_c;
    if constexpr (EPI == kEpiLstm) {
      const float gi = sigmoidf_dev(yx[0] + yh[0] + bias0[0]);
      const float gf = sigmoidf_dev(yx[1] + yh[1] + bias0[1]);
      const float go = sigmoidf_dev(yx[2] + yh[2] + bias0[2]);
      const float gg = tanhf_dev(yx[3] + yh[3] + bias0[3]);
      const float c = fmaf(gf, prev[bt], gi * gg);
      const float h = go * tanhf_dev(c);
      if (bok[bt] && uok) {
        a.c_out[t] = c;
        a.h_out[t] = h;
        if (a.hs_out) a.hs_out[t] = h;
      }
    } else {
      const float rg = sigmoidf_dev(yx[0] + yh[0] + bias0[0] + bias1[0]);
      const float z = sigmoidf_dev(yx[1] + yh[1] + bias0[1] + bias1[1]);
      const float nn = tanhf_dev(fmaf(rg, yh[2] + bias1[2], yx[2] + bias0[2]));
      if (bok[bt] && uok) {
        const float h = fmaf(z, prev[bt] - nn, nn);
        a.h_out[t] = h;
        if (a.hs_out) a.hs_out[t] = h;
      }
    }
  }
  AMQ_PHASE_WHEN(bx == 0 && by == 0, AMQ_PHASE_OF(a), 8, 8);
}

}  // namespace amq
