// Whole batch-1 LSTM sequences in one launch, spread over the chip: the recurrence of Eq. 6 with
// every workgroup keeping its slice of both weight blocks in registers for all time steps.
//
// At batch 1 a step moves a few hundred KB to 3 MB of packed weights and a few KB of state; run
// as two launches per step it is bound by launch gaps and by the cold misses every new kernel
// starts with.  Here a grid of at most 256 workgroups (one per compute unit, all resident) runs
// the whole sequence:
//   - lane = (hidden unit, gate, operand block, 16-byte chunk of the row): a lane holds the KW
//     plane chunks of its row for the whole sequence, and a hidden unit occupies 8 * Gl lanes
//     (Gl = chunks per row rounded up to a power of two, at most 8), so a workgroup of 4 waves
//     owns 4 * 8 / Gl hidden units and the weights are read from memory exactly once;
//   - the inputs x_t do not depend on the recurrence: workgroup g quantizes x_t for t = g, g + G,
//     ... ahead of the loop into a small global table (one grid barrier closes that phase);
//   - per step every workgroup reads h_{t-1} (a few KB), quantizes it itself (4 waves, the shared
//     quantizer core; redundant across workgroups, but it saves a second exchange), forms the
//     pre-activations of its units (xor + popcount, coefficients per lane, DPP sum over the lanes of a
//     unit's gate), applies the cell and publishes its entries of h_t as 8-byte {value, step tag}
//     pairs, each written with one 64-bit device-scope store.  The readers poll the entries they need
//     until all carry the tag of the step: the data is its own arrival signal, so the steps need no
//     barrier and no ordering between separate locations.
// Every wait spins a bounded number of times; if one gives up (the grid was not resident as a whole)
// it raises a flag in the workspace, every workgroup leaves, the state outputs h and c are not
// written and hs is incomplete.  The flag is cleared once per API call, not per launch: the later
// launches of a longer sequence see it and leave at once, and launch_seqg_poison turns whatever was
// derived from hs into NaN.
#include <atomic>

#include "amq_launch.h"
#include "amq_quantize_core.h"

namespace amq {

namespace {

constexpr int kGWaves = 4;
constexpr int kGNJ = 4;                      // vectors of at most 1024 entries: 16 slots over 4 waves
constexpr unsigned kSpinLimit = 1u << 19;    // polls of a wait before giving up
std::atomic<unsigned> g_spin_limit{kSpinLimit};

// Device-scope accesses to the data the workgroups exchange (see grid_barrier).
__device__ __forceinline__ void put_f(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float get_f(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void put_u(uint32_t* p, uint32_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t get_u(const uint32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// All workgroups of the grid meet here.  sync[0] is the give-up flag; the bytes from sync + 1 on
// hold, per workgroup, the low 8 bits of the last epoch it has reached.  Arrival is one plain
// device-scope byte store per workgroup (no read-modify-write, so arrivals do not queue behind
// one another), and the first wave of every workgroup polls all arrival bytes with one 4-byte
// load per lane (256 workgroups = 256 bytes = two cache lines per poll: with a word per
// workgroup the pollers saturated the one memory channel that holds the words).  Workgroups
// are never more than one epoch apart, so a byte equal to the epoch or one above it counts as
// arrived.  Returns false if the barrier was abandoned.
__device__ __forceinline__ bool grid_barrier(unsigned* sync, unsigned epoch, unsigned limit) {
  // Used once per launch (after the inputs have been quantized).  What the workgroups exchange is
  // written and read with device-scope atomic accesses, which go through to the point of coherence
  // on their own.  Ordering: every thread waits for its own exchange stores, the workgroup barrier
  // collects them, and lane 0's arrival store is a release at device scope; the pollers end with an
  // acquire fence at device scope.  (Per step this pair would cost a write-back and an invalidate of
  // the L2 each time, ~40 us measured, which is why the steps exchange self-tagged entries instead.)
  __builtin_amdgcn_s_waitcnt(0);
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __syncthreads();
  int ok = 1;
  if (threadIdx.x < kWave) {
    const int lane = threadIdx.x;
    const int G = gridDim.x;
    unsigned char* arrive = reinterpret_cast<unsigned char*>(sync + 1);
    if (lane == 0)
      __hip_atomic_store(arrive + blockIdx.x, (unsigned char)epoch, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    // this lane watches workgroups 4 * lane .. 4 * lane + 3
    unsigned watch = 0;  // byte mask of the workgroups that exist
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (4 * lane + k < G) watch |= 0xffu << (8 * k);
    unsigned spins = 0;
    for (;;) {
      bool here = true;
      if (watch) {
        const unsigned v = __hip_atomic_load(sync + 1 + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const unsigned d = ((v >> (8 * k)) - epoch) & 0xffu;  // 0 or 1 once that workgroup has arrived
          if ((watch >> (8 * k)) & 1u) here = here && d <= 1u;
        }
      }
      if (__all(here)) break;
      ++spins;
      if (spins > limit) {
        if (lane == 0) __hip_atomic_store(&sync[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        ok = 0;
        break;
      }
      if ((spins & 63u) == 0 && __hip_atomic_load(&sync[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) {
        ok = 0;
        break;
      }
      __builtin_amdgcn_s_sleep(1);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  }
  ok = __syncthreads_and(ok);
  return ok != 0;
}

// The 4 waves of the workgroup quantize one vector of at most 1024 entries together (Alg. 2) and
// leave its planes [KA][wpr] and coefficients [KA] in LDS at `planes` / `coef`.
// Every wave must call this (barriers inside).
// SHARED: the vector is h_{t-1} as the grid publishes it: 8-byte entries {value, tag} written by
// the workgroups that own the hidden units, tag = t.  A lane re-reads its entries until all carry
// the expected tag, so the data itself is the synchronisation: no arrival flags and no separate
// round trip between "everything is there" and "read it".  Returns false if the wait was given up.
template <int KA, bool SHARED>
__device__ __forceinline__ bool quantize_wg(const void* src_v, unsigned tag, unsigned* sync, unsigned limit, int n,
                                            int T, uint32_t* planes, float* coef, double (*sh)[16 * kMaxRed],
                                            int& phase) {
  const int lane = lane_id(), wv = wave_id();
  const int wpr = 4 * ((n + 127) >> 7);
  const int nslots = wpr >> 1;
  const int nj = (nslots + kGWaves - 1) / kGWaves;
  const int base = wv * nj;
  float w[kGNJ];
  int ok = 1;
  if constexpr (SHARED) {
    const unsigned long long* src = static_cast<const unsigned long long*>(src_v);
    unsigned long long v[kGNJ];
    unsigned spins = 0;
    for (;;) {
      bool ready = true;
#pragma unroll
      for (int j = 0; j < kGNJ; ++j) {
        const int e = (base + j) * 64 + lane;
        v[j] = 0ull;
        if (j < nj && e < n) {
          v[j] = __hip_atomic_load(src + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          ready = ready && (unsigned)(v[j] >> 32) == tag;
        }
      }
      if (__all(ready)) break;
      ++spins;
      if (spins > limit) {
        __hip_atomic_store(&sync[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        ok = 0;
        break;
      }
      if ((spins & 63u) == 0 && __hip_atomic_load(&sync[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) {
        ok = 0;
        break;
      }
      __builtin_amdgcn_s_sleep(1);
    }
#pragma unroll
    for (int j = 0; j < kGNJ; ++j) w[j] = __uint_as_float((unsigned)(v[j] & 0xffffffffull));
    ok = __syncthreads_and(ok);
    if (!ok) return false;
  } else {
    const float* src = static_cast<const float*>(src_v);
#pragma unroll
    for (int j = 0; j < kGNJ; ++j) {
      const int e = (base + j) * 64 + lane;
      w[j] = (j < nj && e < n) ? src[e] : 0.0f;
    }
  }
  float alpha[KA];
  unsigned long long mym[KA];
  double q[KA];
#pragma unroll
  for (int i = 0; i < KA; ++i) { alpha[i] = 0.0f; mym[i] = 0ull; q[i] = 0.0; }
  quantize_core<KA, kGNJ, kGWaves>(w, n, base, nj, true, T, true, true, alpha, mym, q, sh, phase);
#pragma unroll
  for (int i = 0; i < KA; ++i) {
    if (lane < nj && base + lane < nslots) reinterpret_cast<unsigned long long*>(planes + i * wpr)[base + lane] = mym[i];
    if (threadIdx.x == 0) coef[i] = alpha[i];
  }
  return true;
}

// Before a launch: clears the arrival bytes and the tags of the published state; the give-up flag only
// for the first launch of an API call.
__global__ void seqg_reset_kernel(unsigned* sync, unsigned long long* hbuf, int H, int clear_flag) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x, nt = gridDim.x * blockDim.x;
  if (t == 0 && clear_flag) sync[0] = 0u;
  for (int i = 1 + t; i < 1 + kSeqGMaxGrid / 4; i += nt) sync[i] = 0u;
  for (int i = t; i < 2 * H; i += nt) hbuf[i] = 0ull;
}

__global__ void seqg_poison_kernel(const unsigned* sync, float* out, long long count) {
  if (*sync == 0u) return;
  const long long nt = (long long)gridDim.x * blockDim.x;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += nt)
    out[i] = __builtin_nanf("");
}

template <int KW, int KA>
__global__ __launch_bounds__(64 * kGWaves) void lstm_seqg_kernel(SeqGArgs a) {
  __shared__ double sh[2][16 * kMaxRed];
  __shared__ __attribute__((aligned(16))) uint32_t xq[KA * 32];  // codes of x_t, [KA][wpr(I)]
  __shared__ __attribute__((aligned(16))) uint32_t hq[KA * 32];  // codes of h_{t-1}
  __shared__ float bx[4], bh[4];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int I = a.I, H = a.H;
  const int cprI = (I + 127) >> 7, cprH = (H + 127) >> 7;
  const int wprI = 4 * cprI;
  const int lg = a.lg, Gl = 1 << lg;        // lanes per (unit, gate, block) row part
  const int UW = 8 >> lg;                   // hidden units per wave
  // lane -> (unit in wave, gate, block, chunk)
  const int c = lane & (Gl - 1);
  const int blk = (lane >> lg) & 1;
  const int gate = (lane >> (lg + 1)) & 3;
  const int uo = lane >> (lg + 3);
  const int unit = (blockIdx.x * kGWaves + wv) * UW + uo;
  const bool uok = unit < H;
  const int row = gate * H + (uok ? unit : 0);
  const int cpr = blk ? cprH : cprI;
  const int nlen = blk ? H : I;
  const bool cok = uok && c < cpr;
  int phase = 0;
  // an earlier launch of the same call gave up: nothing this launch could compute would be valid
  // (one thread reads the flag, so that the whole workgroup takes the same decision)
  __shared__ unsigned gave_up;
  if (threadIdx.x == 0) gave_up = get_u(a.sync);
  __syncthreads();
  if (gave_up != 0u) return;
  const unsigned limit = a.spin_limit;

  // ---- once: this lane's plane chunks and coefficients, the cell lane's bias and state
  uint4 wq[KW];
  float al[KW];
  {
    const uint4* Wp4 = reinterpret_cast<const uint4*>(blk ? a.Whp : a.Wxp);
    const float* alpha = blk ? a.ah : a.ax;
#pragma unroll
    for (int i = 0; i < KW; ++i) {
      const uint4 t4 = Wp4[((long long)i * 4 * H + row) * cpr + (c < cpr ? c : 0)];
      wq[i] = cok ? t4 : make_uint4(0, 0, 0, 0);
      al[i] = alpha[row * KW + i];
    }
  }
  const int left = nlen - 128 * c;
  const float bits = cok ? (float)(left > 128 ? 128 : left) : 0.0f;
  const bool cell = uok && (lane & (8 * Gl - 1)) == 0;   // first lane of the unit applies the cell
  float bs[4], cst = 0.0f, hlast = 0.0f;
#pragma unroll
  for (int g = 0; g < 4; ++g) bs[g] = (cell && a.bias) ? a.bias[g * H + unit] : 0.0f;
  if (cell) {
    cst = a.c[unit];
    hlast = a.h[unit];
  }

  // ---- inputs of all time steps of this launch, quantized ahead by the workgroups in turn
  // (with a.xs null the table has been filled by an earlier launch: the embedding lookup of a
  // language model, whose inputs arrive already quantized)
  for (int t = blockIdx.x; a.xs && t < a.steps; t += gridDim.x) {
    quantize_wg<KA, false>(a.xs + (long long)t * I, 0, a.sync, limit, I, a.T, xq, bx, sh, phase);
    __syncthreads();
    for (int i = tid; i < KA * wprI; i += 64 * kGWaves)
      put_u(a.xq + ((long long)(i / wprI) * a.steps + t) * wprI + i % wprI, xq[i]);
    if (tid < KA) put_f(a.xbeta + t * KA + tid, bx[tid]);
    __syncthreads();
  }
  bool alive = a.xs ? grid_barrier(a.sync, 1, limit) : true;

  // codes of x_0 (KA * wpr(I) <= 128 words: one per thread); those of x_{t+1} are requested while
  // the grid is still working on step t
  uint32_t xnext = 0;
  float bxnext = 0.0f;
  if (alive) {
    if (tid < KA * wprI) xnext = get_u(a.xq + (long long)(tid / wprI) * a.steps * wprI + tid % wprI);
    if (tid < KA) bxnext = get_f(a.xbeta + tid);
  }
  for (int t = 0; t < a.steps && alive; ++t) {
    if (tid < KA * wprI) xq[tid] = xnext;
    if (tid < KA) bx[tid] = bxnext;
    // h_{t-1}: the caller's state at the first step, afterwards what the grid published (tag t)
    if (t == 0) alive = quantize_wg<KA, false>(a.h, 0, a.sync, limit, H, a.T, hq, bh, sh, phase);
    else alive = quantize_wg<KA, true>(a.hbuf + ((t - 1) & 1) * H, (unsigned)t, a.sync, limit, H, a.T, hq, bh, sh, phase);
    if (!alive) break;
    __syncthreads();

    // ---- products of this lane's row chunk, coefficients applied per lane
    const uint4* cq = reinterpret_cast<const uint4*>(blk ? hq : xq);
    const float* beta = blk ? bh : bx;
    float acc = 0.0f;
    {
      uint4 xv[KA];
      float bt[KA];
#pragma unroll
      for (int j = 0; j < KA; ++j) {
        xv[j] = cok ? cq[j * cpr + c] : make_uint4(0, 0, 0, 0);
        bt[j] = beta[j];
      }
#pragma unroll
      for (int i = 0; i < KW; ++i) {
        float inner = 0.0f;
#pragma unroll
        for (int j = 0; j < KA; ++j) inner = fmaf(bt[j], bits - 2.0f * (float)popc4(wq[i], xv[j]), inner);
        acc = fmaf(al[i], inner, acc);
      }
    }
    // sum over the chunks of the row and over the two operand blocks: 2 * Gl adjacent lanes
    const float pre = group_sum(acc, lg + 1);
    // the four gates of a unit sit 2 * Gl lanes apart
    const int ubase = lane & ~(8 * Gl - 1);
    const float p0 = __shfl(pre, ubase, kWave) + bs[0];
    const float p1 = __shfl(pre, ubase + 2 * Gl, kWave) + bs[1];
    const float p2 = __shfl(pre, ubase + 4 * Gl, kWave) + bs[2];
    const float p3 = __shfl(pre, ubase + 6 * Gl, kWave) + bs[3];
    if (cell) {
      const float gi = sigmoidf_dev(p0);
      const float gf = sigmoidf_dev(p1);
      const float go = sigmoidf_dev(p2);
      const float gg = tanhf_dev(p3);
      cst = fmaf(gf, cst, gi * gg);
      hlast = go * tanhf_dev(cst);
      // publish h_t with tag t + 1.  The buffer written here was last read for step t - 1, and no
      // workgroup gets this far before every workgroup has published h_{t-1}, i.e. has finished
      // reading h_{t-2} from this buffer.
      const unsigned long long packed = ((unsigned long long)(unsigned)(t + 1) << 32) | __float_as_uint(hlast);
      __hip_atomic_store(a.hbuf + (t & 1) * H + unit, packed, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (a.hs) a.hs[(long long)t * H + unit] = hlast;
    }
    if (t + 1 < a.steps) {
      if (tid < KA * wprI) xnext = get_u(a.xq + ((long long)(tid / wprI) * a.steps + t + 1) * wprI + tid % wprI);
      if (tid < KA) bxnext = get_f(a.xbeta + (t + 1) * KA + tid);
    }
    __syncthreads();  // xq / hq / bx / bh are rewritten at the top of the next step
  }

  if (alive && cell) {
    a.h[unit] = hlast;
    a.c[unit] = cst;
  }
}

template <int KW, int KA>
hipError_t launch_kk(const SeqGArgs& a, int grid, hipStream_t s) {
  hipLaunchKernelGGL(seqg_reset_kernel, dim3(8), dim3(256), 0, s, a.sync, a.hbuf, a.H, a.first_piece);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((lstm_seqg_kernel<KW, KA>), dim3(grid), dim3(64 * kGWaves), 0, s, a);
  return hipGetLastError();
}

int seqg_lg(int I, int H) {
  const int cpr = ((I > H ? I : H) + 127) / 128;
  int lg = 0;
  while ((1 << lg) < cpr) ++lg;
  return lg;
}

}  // namespace

// Batch 1, 2- or 3-bit codes, vectors of at most 1024 entries; the grid must fit the chip with
// every workgroup resident (at most one per compute unit).
bool lstm_seqg_supported(long long I, long long H, long long B, int k_w, int k_a) {
  if (B != 1 || I > 1024 || H > 1024 || I <= 0 || H <= 0) return false;
  if (k_w < 2 || k_w > 3 || k_a < 2 || k_a > 3) return false;
  const int lg = seqg_lg((int)I, (int)H);
  const int units_per_wg = kGWaves * (8 >> lg);
  return (H + units_per_wg - 1) / units_per_wg <= kSeqGMaxGrid;
}

void set_seqg_spin_limit(unsigned polls) { g_spin_limit.store(polls ? polls : kSpinLimit); }

hipError_t launch_seqg_poison(const unsigned* sync, float* out, long long count, hipStream_t s) {
  if (!out || count <= 0) return hipSuccess;
  const long long blocks = (count + 255) / 256;
  hipLaunchKernelGGL(seqg_poison_kernel, dim3((unsigned)(blocks < 1024 ? blocks : 1024)), dim3(256), 0, s, sync, out,
                     count);
  return hipGetLastError();
}

hipError_t launch_lstm_seqg(SeqGArgs a, int k_w, int k_a, hipStream_t s) {
  a.lg = seqg_lg(a.I, a.H);
  a.spin_limit = g_spin_limit.load();
  const int units_per_wg = kGWaves * (8 >> a.lg);
  const int grid = (a.H + units_per_wg - 1) / units_per_wg;
  if (grid > kSeqGMaxGrid || a.steps > kSeqGMaxSteps) return hipErrorInvalidValue;
  if (k_w == 2 && k_a == 2) return launch_kk<2, 2>(a, grid, s);
  if (k_w == 2 && k_a == 3) return launch_kk<2, 3>(a, grid, s);
  if (k_w == 3 && k_a == 2) return launch_kk<3, 2>(a, grid, s);
  if (k_w == 3 && k_a == 3) return launch_kk<3, 3>(a, grid, s);
  return hipErrorInvalidValue;
}

}  // namespace amq
