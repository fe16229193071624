// C ABI of the library (declared in include/amq.h): argument validation on the host, then
// kernel launches on the caller's stream.  Nothing here allocates or synchronises.
#include "../../include/amq.h"

#include <mutex>

#include "amq_launch.h"

// Scratch memory of amq_lstm_step_static, part of the code object: one copy per GPU the library
// runs on, held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; kernels and host calls take the per-device address it returns.
static __device__ __align__(256) unsigned char scratch[AMQ_STATIC_SCRATCH_BYTES];

#ifdef AMQ_PHASE_TIMING
namespace {
unsigned long long* g_phase_buffer = nullptr;
}
namespace amq {
unsigned long long* phase_buffer() { return g_phase_buffer; }
}  // namespace amq
// Profiling build only: buf = device array of at least 16 * 32 unsigned 64-bit words (or null to stop).
extern "C" void amq_debug_set_phase_buffer(void* buf) { g_phase_buffer = static_cast<unsigned long long*>(buf); }
#endif

namespace {

thread_local int g_last_hip = 0;

int hip_status(hipError_t e) {
  if (e == hipSuccess) return AMQ_OK;
  g_last_hip = (int)e;
  return AMQ_ERR_HIP;
}

// Address of `scratch` on the current device, looked up once per device.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int scratch_of_current_device(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_status(e);
  if (dev < 0 || dev >= kMaxDevices) return AMQ_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_status(e);
    if (!p) return AMQ_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return AMQ_OK;
}

bool bits_ok(int k) { return k >= 1 && k <= AMQ_MAX_BITS; }
bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
size_t up256(size_t b) { return (b + 255) & ~size_t(255); }

// Workspace carving shared by the LSTM / GRU steps.
struct StepWs {
  uint32_t* xp;
  uint32_t* hp;
  float* beta_x;
  float* beta_h;
  float* pre0;
  float* pre1;
  // batch 1 only: scratch of the grid-wide sequence kernel
  unsigned* sync;
  unsigned long long* hbuf;
  uint32_t* xq;
  float* xbeta;
  size_t sync_off;  // byte offset of `sync` in the workspace (SIZE_MAX when the region is absent)
  size_t total;
};

StepWs carve(void* ws, int64_t I, int64_t H, int64_t B, int k_a, int gates, int n_pre) {
  StepWs w;
  size_t off = 0;
  char* base = static_cast<char*>(ws);
  auto take = [&](size_t bytes) {
    char* p = base ? base + off : nullptr;
    off += up256(bytes);
    return p;
  };
  w.xp = reinterpret_cast<uint32_t*>(take(sizeof(uint32_t) * (size_t)k_a * B * amq_wpr(I)));
  w.hp = reinterpret_cast<uint32_t*>(take(sizeof(uint32_t) * (size_t)k_a * B * amq_wpr(H)));
  w.beta_x = reinterpret_cast<float*>(take(sizeof(float) * (size_t)B * k_a));
  w.beta_h = reinterpret_cast<float*>(take(sizeof(float) * (size_t)B * k_a));
  w.pre0 = reinterpret_cast<float*>(take(sizeof(float) * (size_t)B * gates * H));
  w.pre1 = n_pre > 1 ? reinterpret_cast<float*>(take(sizeof(float) * (size_t)B * gates * H)) : nullptr;
  w.sync = nullptr; w.hbuf = nullptr; w.xq = nullptr; w.xbeta = nullptr;
  w.sync_off = SIZE_MAX;
  if (B == 1 && gates == 4) {
    w.sync_off = off;
    w.sync = reinterpret_cast<unsigned*>(take(sizeof(unsigned) * (1 + amq::kSeqGMaxGrid)));
    w.hbuf = reinterpret_cast<unsigned long long*>(take(sizeof(unsigned long long) * 2 * (size_t)H));
    w.xq = reinterpret_cast<uint32_t*>(take(sizeof(uint32_t) * amq::kSeqGMaxSteps * (size_t)k_a * amq_wpr(I)));
    w.xbeta = reinterpret_cast<float*>(take(sizeof(float) * amq::kSeqGMaxSteps * 4));
  }
  w.total = off;
  return w;
}

// Workspace of a batched sequence with given inputs: the step's regions, then what the split step keeps
// between launches -- codes and coefficients of two consecutive inputs, the x-side sums of one step.
struct SeqWs {
  StepWs step;
  uint32_t* xq[2];
  float* xbeta[2];
  float* xsum;
  size_t total;
};

SeqWs carve_seq(void* ws, int64_t I, int64_t H, int64_t B, int k_a, int gates = 4, int n_pre = 1) {
  SeqWs w;
  w.step = carve(ws, I, H, B, k_a, gates, n_pre);
  size_t off = w.step.total;
  char* base = static_cast<char*>(ws);
  auto take = [&](size_t bytes) {
    char* p = base ? base + off : nullptr;
    off += up256(bytes);
    return p;
  };
  for (int i = 0; i < 2; ++i) {
    w.xq[i] = reinterpret_cast<uint32_t*>(take(sizeof(uint32_t) * (size_t)k_a * B * amq_wpr(I)));
    w.xbeta[i] = reinterpret_cast<float*>(take(sizeof(float) * (size_t)B * k_a));
  }
  w.xsum = reinterpret_cast<float*>(take(sizeof(float) * (size_t)B * H * 4));
  w.total = off;
  return w;
}

int check_step(const void* Wxp, const void* ax, const void* Whp, const void* ah, int64_t I, int64_t H,
               int k_w, const void* x, const void* h_prev, int64_t B, int k_a, int T, const void* h_out,
               const void* ws, size_t ws_bytes, size_t need) {
  if (!Wxp || !ax || !Whp || !ah || !x || !h_prev || !h_out || !ws) return AMQ_ERR_INVALID;
  if (!bits_ok(k_w) || !bits_ok(k_a) || T < 0 || I <= 0 || H <= 0 || B <= 0) return AMQ_ERR_INVALID;
  if (!aligned(Wxp, 16) || !aligned(Whp, 16) || !aligned(ws, 256) || ws_bytes < need) return AMQ_ERR_INVALID;
  if (I > AMQ_MAX_QUANT_N || H > AMQ_MAX_QUANT_N || B > (1 << 24)) return AMQ_ERR_UNSUPPORTED;
  return AMQ_OK;
}

// The grid-wide sequence kernel needs all of its (at most kSeqGMaxGrid) workgroups resident at
// once: true when the current device has at least that many compute units.
bool grid_fits_device() {
  static thread_local int cached_dev = -1, cached_cus = 0;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return false;
  if (dev != cached_dev) {
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return false;
    cached_dev = dev;
    cached_cus = cus;
  }
  return cached_cus >= amq::kSeqGMaxGrid;
}

amq::GemmArgs gemm_args(const uint32_t* Wp, const float* alpha, int64_t m, int64_t n, int k_w,
                        const uint32_t* Xp, const float* beta, int64_t batch, int k_a, const float* bias,
                        int accumulate, float* Y) {
  amq::GemmArgs g{};
  g.op.Wp = Wp;
  g.op.alpha = alpha;
  g.op.Xp = Xp;
  g.op.beta = beta;
  g.op.n = (int)n;
  g.m = m;
  g.batch = (int)batch;
  g.k_w = k_w;
  g.k_a = k_a;
  g.bias = bias;
  g.accumulate = accumulate;
  g.Y = Y;
  g.D = nullptr;
  g.lse_part = nullptr;
  g.lse_cap = 0;
  g.groups = 1;
  return g;
}

// Matrix-core product: fp4 kernel when the vectors fit one 1024-entry chunk (its several-tiles-per-wave
// form for large plain products), int8 kernel otherwise.
hipError_t launch_matrix_core(const amq::BmvArgs& b, int k_w, int k_a, int epi, hipStream_t s,
                              int* lse_slots = nullptr) {
  if (epi == amq::kEpiStore && amq::mfma4w_supported(b, k_w, k_a))
    return amq::launch_mfma4w(b, k_w, k_a, s, lse_slots);
  if (epi != amq::kEpiStore && amq::mfma4w_cell_supported(b, k_w, k_a, epi)) {
    if (lse_slots) *lse_slots = 0;
    return amq::launch_mfma4w_cell(b, k_w, k_a, epi, s);
  }
  if (epi != amq::kEpiStore && amq::mfma4_pair_supported(b, k_w, k_a, epi)) {
    if (lse_slots) *lse_slots = 0;
    return amq::launch_mfma4_pair(b, k_w, k_a, epi, s);
  }
  if (amq::mfma4_supported(b, k_w, epi)) return amq::launch_mfma4(b, k_w, k_a, epi, s, lse_slots);
  if (lse_slots) *lse_slots = 0;
  return amq::launch_mfma(b, k_w, k_a, epi, s);
}

amq::BmvArgs store_args(const amq::GemmArgs& g) {
  amq::BmvArgs b{};
  b.blk[0] = amq::BmvBlock{g.op.Wp, g.op.alpha, g.op.Xp, g.op.beta, g.op.n};
  b.m = g.m;
  b.H = 0;
  b.batch = g.batch;
  b.bias0 = g.bias;
  b.accumulate = g.accumulate;
  b.Y = g.Y;
  b.D = g.D;
  b.lse_part = g.lse_part;
  b.lse_cap = g.lse_cap;
  b.groups = g.groups;
  b.g_Wp = g.g_Wp; b.g_alpha = g.g_alpha; b.g_Xp = g.g_Xp; b.g_beta = g.g_beta; b.g_Y = g.g_Y;
  return b;
}

// One quantized product.  Small batches (see kBmvMaxBatchStore): weights-in-registers popcount kernel
// (memory-bound regime).  Larger batches: the matrix-core kernels (dense contraction).  The general
// popcount kernel covers what is left (very long vectors at small batch, grouped products).
// lse_slots (nullable): receives the number of (max, sum) pairs per batch entry the kernel left
// in g.lse_part, or 0 if the kernel that ran does not produce them.
int run_product(const amq::GemmArgs& g, hipStream_t s, int* lse_slots = nullptr) {
  if (lse_slots) *lse_slots = 0;
  if (!g.D && amq::bmv_supported(g.op.n, 0, g.k_a, g.batch, amq::kEpiStore))
    return hip_status(amq::launch_bmv(store_args(g), g.k_w, g.k_a, amq::kEpiStore, s, lse_slots));
  if (g.groups == 1 && amq::mfma_supported(g.batch))
    return hip_status(launch_matrix_core(store_args(g), g.k_w, g.k_a, amq::kEpiStore, s, lse_slots));
  return hip_status(amq::launch_gemm(g, s));
}

int check_product(const void* Wp, int64_t m, int64_t n, int k_w, const void* Xp, int64_t batch, int k_a) {
  if (!Wp || !Xp) return AMQ_ERR_INVALID;
  if (!bits_ok(k_w) || !bits_ok(k_a) || m <= 0 || n <= 0 || batch <= 0) return AMQ_ERR_INVALID;
  if (!aligned(Wp, 16) || !aligned(Xp, 16)) return AMQ_ERR_INVALID;
  if (n > AMQ_MAX_DOT_N || batch > (1 << 24) || m > (1LL << 40)) return AMQ_ERR_UNSUPPORTED;
  return AMQ_OK;
}

int quantize_common(const float* X, int64_t rows, int64_t n, int64_t ld, int k, int T, uint32_t* planes,
                    float* coef, int mode, void* stream) {
  if (!X || !planes || !coef) return AMQ_ERR_INVALID;
  if (!bits_ok(k) || T < 0 || rows <= 0 || n <= 0 || ld < n) return AMQ_ERR_INVALID;
  if (!aligned(planes, 16)) return AMQ_ERR_INVALID;
  if (n > AMQ_MAX_QUANT_N || rows > 0x7fffffffLL) return AMQ_ERR_UNSUPPORTED;
  amq::QuantArgs a{};
  a.seg[0] = amq::QuantSeg{X, ld, (int)n, (int)rows, planes, coef};
  a.seg[1] = amq::QuantSeg{nullptr, 0, 0, 0, nullptr, nullptr};
  a.T = T;
  a.mode = mode;
  return hip_status(amq::launch_quantize(a, k, static_cast<hipStream_t>(stream)));
}

}  // namespace

extern "C" {

int64_t amq_wpr(int64_t n) { return n <= 0 ? 0 : 4 * ((n + 127) / 128); }

const char* amq_version(void) { return "amq 0.1 (gfx950)"; }

const char* amq_status_string(int status) {
  switch (status) {
    case AMQ_OK: return "ok";
    case AMQ_ERR_INVALID: return "invalid argument";
    case AMQ_ERR_UNSUPPORTED: return "unsupported size";
    case AMQ_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

int amq_last_hip_error(void) { return g_last_hip; }

int amq_quantize_weights(const float* W, int64_t rows, int64_t cols, int64_t ld, int k, int T,
                         uint32_t* planes, float* alpha, void* stream) {
  return quantize_common(W, rows, cols, ld, k, T, planes, alpha, amq::kQuantFull, stream);
}

int amq_quantize_activations(const float* X, int64_t batch, int64_t n, int k, int T, uint32_t* planes,
                             float* beta, void* stream) {
  return quantize_common(X, batch, n, n, k, T, planes, beta, amq::kQuantFull, stream);
}

int amq_ls_update(const float* X, int64_t rows, int64_t n, int k, const uint32_t* planes, float* coef,
                  void* stream) {
  return quantize_common(X, rows, n, n, k, 1, const_cast<uint32_t*>(planes), coef, amq::kQuantLsOnly, stream);
}

int amq_bst_assign(const float* X, int64_t rows, int64_t n, int k, const float* coef, uint32_t* planes,
                   void* stream) {
  return quantize_common(X, rows, n, n, k, 1, planes, const_cast<float*>(coef), amq::kQuantBstOnly, stream);
}

int amq_binary_dots(const uint32_t* Wp, int64_t m, int64_t n, int k_w, const uint32_t* Xp, int64_t batch,
                    int k_a, int32_t* D, void* stream) {
  int st = check_product(Wp, m, n, k_w, Xp, batch, k_a);
  if (st != AMQ_OK) return st;
  if (!D) return AMQ_ERR_INVALID;
  // the kernels read coefficients unconditionally; in this integer-only mode they point at any
  // readable memory of sufficient size (the weight planes) and their values are never used
  const float* dummy = reinterpret_cast<const float*>(Wp);
  amq::GemmArgs g = gemm_args(Wp, dummy, m, n, k_w, Xp, dummy, batch, k_a, nullptr, 0, nullptr);
  g.D = D;
  return run_product(g, static_cast<hipStream_t>(stream));
}

int amq_binary_gemm(const uint32_t* Wp, const float* alpha, int64_t m, int64_t n, int k_w,
                    const uint32_t* Xp, const float* beta, int64_t batch, int k_a, const float* bias,
                    int accumulate, float* Y, void* stream) {
  int st = check_product(Wp, m, n, k_w, Xp, batch, k_a);
  if (st != AMQ_OK) return st;
  if (!alpha || !beta || !Y) return AMQ_ERR_INVALID;
  amq::GemmArgs g = gemm_args(Wp, alpha, m, n, k_w, Xp, beta, batch, k_a, bias, accumulate ? 1 : 0, Y);
  return run_product(g, static_cast<hipStream_t>(stream));
}

int amq_binary_gemv(const uint32_t* Wp, const float* alpha, int64_t m, int64_t n, int k_w,
                    const uint32_t* Xp, const float* beta, int k_a, const float* bias, int accumulate,
                    float* Y, void* stream) {
  return amq_binary_gemm(Wp, alpha, m, n, k_w, Xp, beta, 1, k_a, bias, accumulate, Y, stream);
}

int amq_binary_gemv_grouped(int64_t groups, const uint32_t* Wp, const float* alpha, int64_t m, int64_t n,
                            int k_w, const uint32_t* Xp, const float* beta, int k_a, const float* bias,
                            float* Y, void* stream) {
  int st = check_product(Wp, m, n, k_w, Xp, 1, k_a);
  if (st != AMQ_OK) return st;
  if (!alpha || !beta || !Y || groups <= 0) return AMQ_ERR_INVALID;
  if (groups > 65535) return AMQ_ERR_UNSUPPORTED;
  amq::GemmArgs g = gemm_args(Wp, alpha, m, n, k_w, Xp, beta, 1, k_a, bias, 0, Y);
  const int64_t wpr = amq_wpr(n);
  g.groups = (int)groups;
  g.g_Wp = (long long)k_w * m * wpr;
  g.g_alpha = (long long)m * k_w;
  g.g_Xp = (long long)k_a * wpr;
  g.g_beta = k_a;
  g.g_Y = m;
  return run_product(g, static_cast<hipStream_t>(stream));
}

size_t amq_lstm_workspace_bytes(int64_t I, int64_t H, int64_t B, int k_a) {
  if (I <= 0 || H <= 0 || B <= 0 || !bits_ok(k_a)) return 0;
  return carve(nullptr, I, H, B, k_a, 4, 1).total;
}

size_t amq_gru_workspace_bytes(int64_t I, int64_t H, int64_t B, int k_a) {
  if (I <= 0 || H <= 0 || B <= 0 || !bits_ok(k_a)) return 0;
  return carve(nullptr, I, H, B, k_a, 3, 2).total;
}

// Products + epilogue + cell in one launch, given quantized operands.  Returns -1 if no fused
// kernel takes this shape (the caller then uses the unfused path, which needs a workspace).
static amq::BmvArgs lstm_args(const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp, const float* alpha_h,
                              int64_t I, int64_t H, const float* bias, const uint32_t* Xp, const float* beta_x,
                              const uint32_t* Hp, const float* beta_h, const float* c_prev, int64_t B, float* h_out,
                              float* c_out, float* hs_out) {
  amq::BmvArgs b{};
  b.blk[0] = amq::BmvBlock{Wxp, alpha_x, Xp, beta_x, (int)I};
  b.blk[1] = amq::BmvBlock{Whp, alpha_h, Hp, beta_h, (int)H};
  b.m = 4 * H;
  b.H = H;
  b.batch = (int)B;
  b.bias0 = bias;
  b.c_prev = c_prev;
  b.h_out = h_out;
  b.c_out = c_out;
  b.hs_out = hs_out;
  b.groups = 1;
  return b;
}

static int lstm_fused_launch(const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp,
                             const float* alpha_h, int64_t I, int64_t H, int k_w, const float* bias,
                             const uint32_t* Xp, const float* beta_x, const uint32_t* Hp, const float* beta_h,
                             const float* c_prev, int64_t B, int k_a, float* h_out, float* c_out,
                             float* hs_out, hipStream_t s) {
  const amq::BmvArgs b = lstm_args(Wxp, alpha_x, Whp, alpha_h, I, H, bias, Xp, beta_x, Hp, beta_h, c_prev, B, h_out,
                                   c_out, hs_out);
  if (amq::bmv_supported((int)I, (int)H, k_a, B, amq::kEpiLstm))
    return hip_status(amq::launch_bmv(b, k_w, k_a, amq::kEpiLstm, s));
  if (amq::mfma_supported(B))
    return hip_status(launch_matrix_core(b, k_w, k_a, amq::kEpiLstm, s));
  return -1;
}

static int lstm_step_launch(const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp,
                            const float* alpha_h, int64_t I, int64_t H, int k_w, const float* bias,
                            const float* x, const float* h_prev, const float* c_prev, int64_t B, int k_a,
                            int T, float* h_out, float* c_out, float* hs_out, const StepWs& w,
                            hipStream_t s) {
  amq::QuantArgs q{};
  q.seg[0] = amq::QuantSeg{x, I, (int)I, (int)B, w.xp, w.beta_x};
  q.seg[1] = amq::QuantSeg{h_prev, H, (int)H, (int)B, w.hp, w.beta_h};
  q.T = T;
  q.mode = amq::kQuantFull;
  int st = hip_status(amq::launch_quantize(q, k_a, s));
  if (st != AMQ_OK) return st;
  st = lstm_fused_launch(Wxp, alpha_x, Whp, alpha_h, I, H, k_w, bias, w.xp, w.beta_x, w.hp, w.beta_h, c_prev,
                         B, k_a, h_out, c_out, hs_out, s);
  if (st >= 0) return st;
  amq::GemmArgs gx = gemm_args(Wxp, alpha_x, 4 * H, I, k_w, w.xp, w.beta_x, B, k_a, bias, 0, w.pre0);
  st = run_product(gx, s);
  if (st != AMQ_OK) return st;
  amq::GemmArgs gh = gemm_args(Whp, alpha_h, 4 * H, H, k_w, w.hp, w.beta_h, B, k_a, nullptr, 1, w.pre0);
  st = run_product(gh, s);
  if (st != AMQ_OK) return st;
  return hip_status(amq::launch_lstm_pointwise(w.pre0, c_prev, h_out, c_out, hs_out, B, H, s));
}

int amq_lstm_step_packed_grouped(int64_t groups, const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp,
                                 const float* alpha_h, int64_t I, int64_t H, int k_w, const float* bias,
                                 const uint32_t* Xp, const float* beta_x, const uint32_t* Hp, const float* beta_h,
                                 const float* c_prev, int k_a, float* h_out, float* c_out, void* stream) {
  if (!Wxp || !alpha_x || !Whp || !alpha_h || !Xp || !beta_x || !Hp || !beta_h || !c_prev || !h_out || !c_out)
    return AMQ_ERR_INVALID;
  if (!bits_ok(k_w) || !bits_ok(k_a) || I <= 0 || H <= 0 || groups <= 0) return AMQ_ERR_INVALID;
  if (!aligned(Wxp, 16) || !aligned(Whp, 16) || !aligned(Xp, 16) || !aligned(Hp, 16)) return AMQ_ERR_INVALID;
  if (groups > 65535 || !amq::bmv_supported((int)I, (int)H, k_a, 1, amq::kEpiLstm)) return AMQ_ERR_UNSUPPORTED;
  amq::BmvArgs b{};
  b.blk[0] = amq::BmvBlock{Wxp, alpha_x, Xp, beta_x, (int)I};
  b.blk[1] = amq::BmvBlock{Whp, alpha_h, Hp, beta_h, (int)H};
  b.m = 4 * H;
  b.H = H;
  b.batch = 1;
  b.bias0 = bias;
  b.c_prev = c_prev;
  b.h_out = h_out;
  b.c_out = c_out;
  b.groups = (int)groups;
  b.g_Wp = (long long)k_w * 4 * H * amq_wpr(I);
  b.g_Wp1 = (long long)k_w * 4 * H * amq_wpr(H);
  b.g_alpha = b.g_alpha1 = 4 * H * k_w;
  b.g_Xp = (long long)k_a * amq_wpr(I);
  b.g_Xp1 = (long long)k_a * amq_wpr(H);
  b.g_beta = b.g_beta1 = k_a;
  b.g_state = H;
  return hip_status(amq::launch_bmv(b, k_w, k_a, amq::kEpiLstm, static_cast<hipStream_t>(stream)));
}

int amq_stream_read_probe(const void* buf, size_t bytes, void* sink, void* stream) {
  if (!buf || !sink || bytes == 0 || (bytes & 15) || !aligned(buf, 16) || !aligned(sink, 8)) return AMQ_ERR_INVALID;
  return hip_status(amq::launch_stream_read(buf, bytes, static_cast<unsigned long long*>(sink),
                                            static_cast<hipStream_t>(stream)));
}

int amq_lstm_step_packed(const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp, const float* alpha_h,
                         int64_t I, int64_t H, int k_w, const float* bias, const uint32_t* Xp,
                         const float* beta_x, const uint32_t* Hp, const float* beta_h, const float* c_prev,
                         int64_t B, int k_a, float* h_out, float* c_out, void* stream) {
  if (!Wxp || !alpha_x || !Whp || !alpha_h || !Xp || !beta_x || !Hp || !beta_h || !c_prev || !h_out || !c_out)
    return AMQ_ERR_INVALID;
  if (!bits_ok(k_w) || !bits_ok(k_a) || I <= 0 || H <= 0 || B <= 0) return AMQ_ERR_INVALID;
  if (!aligned(Wxp, 16) || !aligned(Whp, 16) || !aligned(Xp, 16) || !aligned(Hp, 16)) return AMQ_ERR_INVALID;
  if (I > AMQ_MAX_QUANT_N || H > AMQ_MAX_QUANT_N || B > (1 << 24)) return AMQ_ERR_UNSUPPORTED;
  int st = lstm_fused_launch(Wxp, alpha_x, Whp, alpha_h, I, H, k_w, bias, Xp, beta_x, Hp, beta_h, c_prev, B, k_a,
                             h_out, c_out, nullptr, static_cast<hipStream_t>(stream));
  return st >= 0 ? st : AMQ_ERR_UNSUPPORTED;
}

int amq_lstm_step(const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp, const float* alpha_h,
                  int64_t I, int64_t H, int k_w, const float* bias, const float* x, const float* h_prev,
                  const float* c_prev, int64_t B, int k_a, int T, float* h_out, float* c_out,
                  void* workspace, size_t workspace_bytes, void* stream) {
  if (!c_prev || !c_out) return AMQ_ERR_INVALID;
  const size_t need = (I > 0 && H > 0 && B > 0 && bits_ok(k_a)) ? carve(nullptr, I, H, B, k_a, 4, 1).total : 0;
  int st = check_step(Wxp, alpha_x, Whp, alpha_h, I, H, k_w, x, h_prev, B, k_a, T, h_out, workspace,
                      workspace_bytes, need);
  if (st != AMQ_OK) return st;
  StepWs w = carve(workspace, I, H, B, k_a, 4, 1);
  return lstm_step_launch(Wxp, alpha_x, Whp, alpha_h, I, H, k_w, bias, x, h_prev, c_prev, B, k_a, T, h_out,
                          c_out, nullptr, w, static_cast<hipStream_t>(stream));
}

int amq_lstm_step_static(const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp, const float* alpha_h,
                         int64_t I, int64_t H, int k_w, const float* bias, const float* x, const float* h_prev,
                         const float* c_prev, int64_t B, int k_a, int T, float* h_out, float* c_out, void* stream) {
  if (!c_prev || !c_out) return AMQ_ERR_INVALID;
  const size_t need = (I > 0 && H > 0 && B > 0 && bits_ok(k_a)) ? carve(nullptr, I, H, B, k_a, 4, 1).total : 0;
  // (validated against a stand-in workspace address: the real one is looked up only for sizes that fit)
  int st = check_step(Wxp, alpha_x, Whp, alpha_h, I, H, k_w, x, h_prev, B, k_a, T, h_out,
                      reinterpret_cast<const void*>(uintptr_t(256)), need, need);
  if (st != AMQ_OK) return st;
  if (need > AMQ_STATIC_SCRATCH_BYTES) return AMQ_ERR_UNSUPPORTED;
  void* ws = nullptr;
  st = scratch_of_current_device(&ws);
  if (st != AMQ_OK) return st;
  // every region of the scratch that a step reads is written earlier in the same step (codes and
  // coefficients by the quantizer, pre-activations by the first product), so nothing is cleared
  StepWs w = carve(ws, I, H, B, k_a, 4, 1);
  return lstm_step_launch(Wxp, alpha_x, Whp, alpha_h, I, H, k_w, bias, x, h_prev, c_prev, B, k_a, T, h_out,
                          c_out, nullptr, w, static_cast<hipStream_t>(stream));
}

size_t amq_lstm_sequence_workspace_bytes(int64_t I, int64_t H, int64_t B, int k_a) {
  if (I <= 0 || H <= 0 || B <= 0 || !bits_ok(k_a)) return 0;
  return carve_seq(nullptr, I, H, B, k_a).total;
}

size_t amq_lstm_sequence_flag_offset(int64_t I, int64_t H, int64_t B, int k_a) {
  if (I <= 0 || H <= 0 || B <= 0 || !bits_ok(k_a)) return SIZE_MAX;
  return carve(nullptr, I, H, B, k_a, 4, 1).sync_off;
}

void amq_debug_set_sequence_spin_limit(unsigned polls) { amq::set_seqg_spin_limit(polls); }

int amq_lstm_sequence(const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp, const float* alpha_h,
                      int64_t I, int64_t H, int k_w, const float* bias, const float* xs, int64_t steps,
                      float* h, float* c, int64_t B, int k_a, int T, float* hs, void* workspace,
                      size_t workspace_bytes, void* stream) {
  if (!c || steps <= 0) return AMQ_ERR_INVALID;
  const size_t need = (I > 0 && H > 0 && B > 0 && bits_ok(k_a)) ? carve(nullptr, I, H, B, k_a, 4, 1).total : 0;
  int st = check_step(Wxp, alpha_x, Whp, alpha_h, I, H, k_w, xs, h, B, k_a, T, h, workspace, workspace_bytes,
                      need);
  if (st != AMQ_OK) return st;
  if (steps < (1 << 30) && amq::lstm_seqg_supported(I, H, B, k_w, k_a) && grid_fits_device()) {
    // batch 1: the whole sequence (in pieces of at most kSeqGMaxSteps steps) in one launch over the
    // chip, weights resident in registers
    StepWs w = carve(workspace, I, H, B, k_a, 4, 1);
    for (int64_t t0 = 0; t0 < steps; t0 += amq::kSeqGMaxSteps) {
      const int n = (int)(steps - t0 < amq::kSeqGMaxSteps ? steps - t0 : amq::kSeqGMaxSteps);
      amq::SeqGArgs q{Wxp, alpha_x, Whp, alpha_h, (int)I, (int)H, bias, xs + t0 * I, n, h, c,
                      hs ? hs + t0 * H : nullptr, T, 0, w.sync, w.hbuf, w.xq, w.xbeta, t0 == 0, 0};
      st = hip_status(amq::launch_lstm_seqg(q, k_w, k_a, static_cast<hipStream_t>(stream)));
      if (st != AMQ_OK) return st;
      // a launch that gave up (or found the flag of an earlier one) leaves its rows of hs as NaN
      if (hs) {
        st = hip_status(amq::launch_seqg_poison(w.sync, hs + t0 * H, (long long)n * H, static_cast<hipStream_t>(stream)));
        if (st != AMQ_OK) return st;
      }
    }
    return AMQ_OK;
  }
  StepWs w = carve(workspace, I, H, B, k_a, 4, 1);
  hipStream_t s = static_cast<hipStream_t>(stream);
  {
    // The inputs are all given, so W_x x_t is taken off the recurrent chain where the shape allows and the
    // workspace has room (amq_lstm_sequence_workspace_bytes): per step a front launch (quantize h_{t-1} and,
    // in its shadow, quantize x_{t+1} and form the x-side sums of step t from the codes of x_t) and a back
    // launch (h-side sums + stored x-side sums + cell).  The first step has no codes of x_0 yet: its front
    // launch quantizes h, x_0 and x_1 and its back launch is the whole-step kernel.  Same results as the
    // per-step path, bit for bit.
    const SeqWs sw = carve_seq(workspace, I, H, B, k_a);
    const amq::BmvArgs probe = lstm_args(Wxp, alpha_x, Whp, alpha_h, I, H, bias, sw.xq[0], sw.xbeta[0], w.hp, w.beta_h,
                                         c, B, h, c, nullptr);
    if (workspace_bytes >= sw.total && amq::step_split_supported(probe, k_w, k_a, amq::kEpiLstm)) {
      auto step_args = [&](int64_t t) {
        amq::BmvArgs b = probe;
        b.blk[0].Xp = sw.xq[t % 2];
        b.blk[0].beta = sw.xbeta[t % 2];
        b.Y = sw.xsum;
        b.hs_out = hs ? hs + t * B * H : nullptr;
        return b;
      };
      auto x_seg = [&](int64_t u) {
        return amq::QuantSeg{xs + u * B * I, I, (int)I, (int)B, sw.xq[u % 2], sw.xbeta[u % 2]};
      };
      for (int64_t t = 0; t < steps; ++t) {
        amq::QuantArgs q{}, q2{};
        q.seg[0] = amq::QuantSeg{h, H, (int)H, (int)B, w.hp, w.beta_h};
        q.T = q2.T = T;
        q.mode = q2.mode = amq::kQuantFull;
        const amq::BmvArgs b = step_args(t);
        if (t == 0) {
          q.seg[1] = x_seg(0);
          if (steps > 1) q2.seg[0] = x_seg(1);
          st = hip_status(amq::launch_step_front(q, steps > 1 ? &q2 : nullptr, nullptr, k_w, k_a, amq::kEpiLstm, s));
          if (st != AMQ_OK) return st;
          st = hip_status(amq::launch_mfma4_pair(b, k_w, k_a, amq::kEpiLstm, s));
        } else {
          if (t + 1 < steps) q.seg[1] = x_seg(t + 1);
          st = hip_status(amq::launch_step_front(q, nullptr, &b, k_w, k_a, amq::kEpiLstm, s));
          if (st != AMQ_OK) return st;
          st = hip_status(amq::launch_step_back(b, k_w, k_a, amq::kEpiLstm, s));
        }
        if (st != AMQ_OK) return st;
      }
      return AMQ_OK;
    }
  }
  for (int64_t t = 0; t < steps; ++t) {
    st = lstm_step_launch(Wxp, alpha_x, Whp, alpha_h, I, H, k_w, bias, xs + t * B * I, h, c, B, k_a, T, h, c,
                          hs ? hs + t * B * H : nullptr, w, s);
    if (st != AMQ_OK) return st;
  }
  return AMQ_OK;
}

int amq_debug_lstm_split_half(const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp, const float* alpha_h,
                              int64_t I, int64_t H, int k_w, const float* bias, const float* x_next, float* h, float* c,
                              int64_t B, int k_a, int T, void* workspace, size_t workspace_bytes, int half,
                              void* stream) {
  if (!c || !x_next || (half != 0 && half != 1)) return AMQ_ERR_INVALID;
  const size_t need = (I > 0 && H > 0 && B > 0 && bits_ok(k_a)) ? carve_seq(nullptr, I, H, B, k_a).total : 0;
  int st = check_step(Wxp, alpha_x, Whp, alpha_h, I, H, k_w, x_next, h, B, k_a, T, h, workspace, workspace_bytes, need);
  if (st != AMQ_OK) return st;
  const SeqWs sw = carve_seq(workspace, I, H, B, k_a);
  amq::BmvArgs b = lstm_args(Wxp, alpha_x, Whp, alpha_h, I, H, bias, sw.xq[0], sw.xbeta[0], sw.step.hp, sw.step.beta_h, c,
                             B, h, c, nullptr);
  b.Y = sw.xsum;
  if (!amq::step_split_supported(b, k_w, k_a, amq::kEpiLstm)) return AMQ_ERR_UNSUPPORTED;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (half == 1) return hip_status(amq::launch_step_back(b, k_w, k_a, amq::kEpiLstm, s));
  amq::QuantArgs q{};
  q.seg[0] = amq::QuantSeg{h, H, (int)H, (int)B, sw.step.hp, sw.step.beta_h};
  q.seg[1] = amq::QuantSeg{x_next, I, (int)I, (int)B, sw.xq[1], sw.xbeta[1]};
  q.T = T;
  q.mode = amq::kQuantFull;
  return hip_status(amq::launch_step_front(q, nullptr, &b, k_w, k_a, amq::kEpiLstm, s));
}

static amq::BmvArgs gru_args(const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp, const float* alpha_h,
                             int64_t I, int64_t H, const float* bias_x, const float* bias_h, const uint32_t* Xp,
                             const float* beta_x, const uint32_t* Hp, const float* beta_h, const float* h_prev,
                             int64_t B, float* h_out) {
  amq::BmvArgs b{};
  b.blk[0] = amq::BmvBlock{Wxp, alpha_x, Xp, beta_x, (int)I};
  b.blk[1] = amq::BmvBlock{Whp, alpha_h, Hp, beta_h, (int)H};
  b.m = 3 * H;
  b.H = H;
  b.batch = (int)B;
  b.bias0 = bias_x;
  b.bias1 = bias_h;
  b.h_prev = h_prev;
  b.h_out = h_out;
  b.groups = 1;
  return b;
}

// The launches of one GRU step on a carved workspace (arguments already validated).
static int gru_step_launch(const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp, const float* alpha_h,
                           int64_t I, int64_t H, int k_w, const float* bias_x, const float* bias_h, const float* x,
                           const float* h_prev, int64_t B, int k_a, int T, float* h_out, const StepWs& w,
                           hipStream_t s) {
  amq::QuantArgs q{};
  q.seg[0] = amq::QuantSeg{x, I, (int)I, (int)B, w.xp, w.beta_x};
  q.seg[1] = amq::QuantSeg{h_prev, H, (int)H, (int)B, w.hp, w.beta_h};
  q.T = T;
  q.mode = amq::kQuantFull;
  int st = hip_status(amq::launch_quantize(q, k_a, s));
  if (st != AMQ_OK) return st;
  const amq::BmvArgs b = gru_args(Wxp, alpha_x, Whp, alpha_h, I, H, bias_x, bias_h, w.xp, w.beta_x, w.hp, w.beta_h,
                                  h_prev, B, h_out);
  if (amq::bmv_supported((int)I, (int)H, k_a, B, amq::kEpiGru))
    return hip_status(amq::launch_bmv(b, k_w, k_a, amq::kEpiGru, s));
  if (amq::mfma_supported(B)) return hip_status(launch_matrix_core(b, k_w, k_a, amq::kEpiGru, s));
  amq::GemmArgs gx = gemm_args(Wxp, alpha_x, 3 * H, I, k_w, w.xp, w.beta_x, B, k_a, bias_x, 0, w.pre0);
  st = run_product(gx, s);
  if (st != AMQ_OK) return st;
  amq::GemmArgs gh = gemm_args(Whp, alpha_h, 3 * H, H, k_w, w.hp, w.beta_h, B, k_a, bias_h, 0, w.pre1);
  st = run_product(gh, s);
  if (st != AMQ_OK) return st;
  return hip_status(amq::launch_gru_pointwise(w.pre0, w.pre1, h_prev, h_out, B, H, s));
}

int amq_gru_step(const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp, const float* alpha_h,
                 int64_t I, int64_t H, int k_w, const float* bias_x, const float* bias_h, const float* x,
                 const float* h_prev, int64_t B, int k_a, int T, float* h_out, void* workspace,
                 size_t workspace_bytes, void* stream) {
  const size_t need = (I > 0 && H > 0 && B > 0 && bits_ok(k_a)) ? carve(nullptr, I, H, B, k_a, 3, 2).total : 0;
  int st = check_step(Wxp, alpha_x, Whp, alpha_h, I, H, k_w, x, h_prev, B, k_a, T, h_out, workspace,
                      workspace_bytes, need);
  if (st != AMQ_OK) return st;
  const StepWs w = carve(workspace, I, H, B, k_a, 3, 2);
  return gru_step_launch(Wxp, alpha_x, Whp, alpha_h, I, H, k_w, bias_x, bias_h, x, h_prev, B, k_a, T, h_out, w,
                         static_cast<hipStream_t>(stream));
}

size_t amq_gru_sequence_workspace_bytes(int64_t I, int64_t H, int64_t B, int k_a) {
  if (I <= 0 || H <= 0 || B <= 0 || !bits_ok(k_a)) return 0;
  return carve_seq(nullptr, I, H, B, k_a, 3, 2).total;
}

int amq_gru_sequence(const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp, const float* alpha_h,
                     int64_t I, int64_t H, int k_w, const float* bias_x, const float* bias_h, const float* xs,
                     int64_t steps, float* h, int64_t B, int k_a, int T, float* hs, void* workspace,
                     size_t workspace_bytes, void* stream) {
  if (steps <= 0) return AMQ_ERR_INVALID;
  const size_t need = (I > 0 && H > 0 && B > 0 && bits_ok(k_a)) ? carve(nullptr, I, H, B, k_a, 3, 2).total : 0;
  int st = check_step(Wxp, alpha_x, Whp, alpha_h, I, H, k_w, xs, h, B, k_a, T, h, workspace, workspace_bytes, need);
  if (st != AMQ_OK) return st;
  if (steps >= (1 << 30)) return AMQ_ERR_UNSUPPORTED;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const StepWs w = carve(workspace, I, H, B, k_a, 3, 2);
  const SeqWs sw = carve_seq(workspace, I, H, B, k_a, 3, 2);
  const amq::BmvArgs probe = gru_args(Wxp, alpha_x, Whp, alpha_h, I, H, bias_x, bias_h, sw.xq[0], sw.xbeta[0], w.hp,
                                      w.beta_h, h, B, h);
  if (workspace_bytes >= sw.total && amq::step_split_supported(probe, k_w, k_a, amq::kEpiGru)) {
    // As in amq_lstm_sequence: the inputs are given, so W_x x_t leaves the recurrent chain.  Front launch of
    // step t: quantize h_{t-1}, quantize x_{t+1}, x-side sums of step t; back launch: h-side sums + the
    // stored x-side sums + cell, h updated in place.  The first step quantizes h, x_0 and x_1 and runs the
    // whole-step kernel.  Same results as amq_gru_step called step by step, bit for bit.
    auto x_seg = [&](int64_t u) {
      return amq::QuantSeg{xs + u * B * I, I, (int)I, (int)B, sw.xq[u % 2], sw.xbeta[u % 2]};
    };
    for (int64_t t = 0; t < steps; ++t) {
      amq::BmvArgs b = probe;
      b.blk[0].Xp = sw.xq[t % 2];
      b.blk[0].beta = sw.xbeta[t % 2];
      b.Y = sw.xsum;
      b.hs_out = hs ? hs + t * B * H : nullptr;
      amq::QuantArgs q{}, q2{};
      q.seg[0] = amq::QuantSeg{h, H, (int)H, (int)B, w.hp, w.beta_h};
      q.T = q2.T = T;
      q.mode = q2.mode = amq::kQuantFull;
      if (t == 0) {
        q.seg[1] = x_seg(0);
        if (steps > 1) q2.seg[0] = x_seg(1);
        st = hip_status(amq::launch_step_front(q, steps > 1 ? &q2 : nullptr, nullptr, k_w, k_a, amq::kEpiGru, s));
        if (st != AMQ_OK) return st;
        st = hip_status(amq::launch_mfma4_pair(b, k_w, k_a, amq::kEpiGru, s));
      } else {
        if (t + 1 < steps) q.seg[1] = x_seg(t + 1);
        st = hip_status(amq::launch_step_front(q, nullptr, &b, k_w, k_a, amq::kEpiGru, s));
        if (st != AMQ_OK) return st;
        st = hip_status(amq::launch_step_back(b, k_w, k_a, amq::kEpiGru, s));
      }
      if (st != AMQ_OK) return st;
    }
    return AMQ_OK;
  }
  // step-by-step launches; with hs given each step writes its slot and reads the one before, and the last
  // slot is copied to h at the end
  for (int64_t t = 0; t < steps; ++t) {
    const float* prev = (hs && t > 0) ? hs + (t - 1) * B * H : h;
    float* out = hs ? hs + t * B * H : h;
    st = gru_step_launch(Wxp, alpha_x, Whp, alpha_h, I, H, k_w, bias_x, bias_h, xs + t * B * I, prev, B, k_a, T, out, w,
                         s);
    if (st != AMQ_OK) return st;
  }
  if (hs) return hip_status(hipMemcpyAsync(h, hs + (steps - 1) * B * H, sizeof(float) * (size_t)B * H,
                                           hipMemcpyDeviceToDevice, s));
  return AMQ_OK;
}

// Workspace of the reset-before GRU step: that of amq_gru_step, then a third pre-activation
// buffer and g = r * h_prev.
struct GruRbWs {
  StepWs base;
  float* pre2;
  float* g;
  size_t total;
};
static GruRbWs carve_gru_rb(void* ws, int64_t I, int64_t H, int64_t B, int k_a) {
  GruRbWs w;
  w.base = carve(ws, I, H, B, k_a, 3, 2);
  char* p = static_cast<char*>(ws);
  size_t off = w.base.total;
  w.pre2 = reinterpret_cast<float*>(p ? p + off : nullptr);
  off += up256(sizeof(float) * (size_t)B * 3 * H);
  w.g = reinterpret_cast<float*>(p ? p + off : nullptr);
  off += up256(sizeof(float) * (size_t)B * H);
  w.total = off;
  return w;
}

size_t amq_gru_reset_before_workspace_bytes(int64_t I, int64_t H, int64_t B, int k_a) {
  if (I <= 0 || H <= 0 || B <= 0 || !bits_ok(k_a)) return 0;
  return carve_gru_rb(nullptr, I, H, B, k_a).total;
}

int amq_gru_step_reset_before(const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp, const float* alpha_h,
                              int64_t I, int64_t H, int k_w, const float* bias_x, const float* bias_h,
                              const float* x, const float* h_prev, int64_t B, int k_a, int T, float* h_out,
                              float* g_out, void* workspace, size_t workspace_bytes, void* stream) {
  const size_t need = (I > 0 && H > 0 && B > 0 && bits_ok(k_a)) ? carve_gru_rb(nullptr, I, H, B, k_a).total : 0;
  int st = check_step(Wxp, alpha_x, Whp, alpha_h, I, H, k_w, x, h_prev, B, k_a, T, h_out, workspace,
                      workspace_bytes, need);
  if (st != AMQ_OK) return st;
  GruRbWs w = carve_gru_rb(workspace, I, H, B, k_a);
  if (g_out) w.g = g_out;
  hipStream_t s = static_cast<hipStream_t>(stream);
  amq::QuantArgs q{};
  q.seg[0] = amq::QuantSeg{x, I, (int)I, (int)B, w.base.xp, w.base.beta_x};
  q.seg[1] = amq::QuantSeg{h_prev, H, (int)H, (int)B, w.base.hp, w.base.beta_h};
  q.T = T;
  q.mode = amq::kQuantFull;
  st = hip_status(amq::launch_quantize(q, k_a, s));
  if (st != AMQ_OK) return st;
  amq::GemmArgs gx = gemm_args(Wxp, alpha_x, 3 * H, I, k_w, w.base.xp, w.base.beta_x, B, k_a, bias_x, 0, w.base.pre0);
  st = run_product(gx, s);
  if (st != AMQ_OK) return st;
  amq::GemmArgs gh = gemm_args(Whp, alpha_h, 3 * H, H, k_w, w.base.hp, w.base.beta_h, B, k_a, bias_h, 0, w.base.pre1);
  st = run_product(gh, s);
  if (st != AMQ_OK) return st;
  st = hip_status(amq::launch_gru_rb_reset(w.base.pre0, w.base.pre1, h_prev, w.g, B, H, s));
  if (st != AMQ_OK) return st;
  // g = r * h_prev is quantized on line like any activation (its codes reuse the buffer of h's),
  // and the whole hidden-side product is formed again; only its candidate rows are used
  amq::QuantArgs qg{};
  qg.seg[0] = amq::QuantSeg{w.g, H, (int)H, (int)B, w.base.hp, w.base.beta_h};
  qg.T = T;
  qg.mode = amq::kQuantFull;
  st = hip_status(amq::launch_quantize(qg, k_a, s));
  if (st != AMQ_OK) return st;
  amq::GemmArgs gg = gemm_args(Whp, alpha_h, 3 * H, H, k_w, w.base.hp, w.base.beta_h, B, k_a, bias_h, 0, w.pre2);
  st = run_product(gg, s);
  if (st != AMQ_OK) return st;
  return hip_status(amq::launch_gru_rb_final(w.base.pre0, w.base.pre1, w.pre2, h_prev, h_out, B, H, s));
}

int amq_quantize_weights_ex(const float* W, int64_t rows, int64_t cols, int64_t ld, int k, int T, int flags,
                            uint32_t* planes, float* alpha, void* stream) {
  if (flags & ~AMQ_QUANT_FINAL_LS) return AMQ_ERR_INVALID;
  int st = quantize_common(W, rows, cols, ld, k, T, planes, alpha, amq::kQuantFull, stream);
  if (st != AMQ_OK || !(flags & AMQ_QUANT_FINAL_LS)) return st;
  // the trailing coefficient update is the staged Eq. 5 pass on the codes just written (a second
  // launch, so that the main kernel carries no code for it)
  return quantize_common(W, rows, cols, ld, k, 1, planes, alpha, amq::kQuantLsOnly, stream);
}

int amq_dequantize(const uint32_t* planes, const float* alpha, int64_t rows, int64_t cols, int k, float* out,
                   int64_t ld_out, void* stream) {
  if (!planes || !alpha || !out) return AMQ_ERR_INVALID;
  if (!bits_ok(k) || rows <= 0 || cols <= 0 || ld_out < cols) return AMQ_ERR_INVALID;
  if (cols > (1 << 30) || rows > (1LL << 33)) return AMQ_ERR_UNSUPPORTED;
  return hip_status(amq::launch_dequantize(planes, alpha, rows, (int)cols, k, out, ld_out,
                                           static_cast<hipStream_t>(stream)));
}

int amq_clip(float* w, int64_t n, float lo, float hi, void* stream) {
  if (!w || n <= 0 || !(lo <= hi)) return AMQ_ERR_INVALID;
  if (n > (1LL << 39)) return AMQ_ERR_UNSUPPORTED;
  return hip_status(amq::launch_clip(w, n, lo, hi, static_cast<hipStream_t>(stream)));
}

int amq_quantize_refined_greedy(const float* W, int64_t rows, int64_t cols, int64_t ld, int k, uint32_t* planes,
                                float* alpha, void* stream) {
  if (!W || !planes || !alpha) return AMQ_ERR_INVALID;
  if (!bits_ok(k) || rows <= 0 || cols <= 0 || ld < cols) return AMQ_ERR_INVALID;
  if (!aligned(planes, 16)) return AMQ_ERR_INVALID;
  if (cols > AMQ_MAX_QUANT_N || rows > 0x7fffffffLL) return AMQ_ERR_UNSUPPORTED;
  return hip_status(amq::launch_refined_greedy(W, ld, (int)cols, (int)rows, k, planes, alpha,
                                               static_cast<hipStream_t>(stream)));
}

int amq_quantize_ternary(const float* W, int64_t rows, int64_t cols, int64_t ld, int T, uint32_t* planes,
                         float* alpha, void* stream) {
  if (!W || !planes || !alpha) return AMQ_ERR_INVALID;
  if (T < 0 || rows <= 0 || cols <= 0 || ld < cols) return AMQ_ERR_INVALID;
  if (!aligned(planes, 16)) return AMQ_ERR_INVALID;
  if (cols > AMQ_MAX_QUANT_N || rows > 0x7fffffffLL) return AMQ_ERR_UNSUPPORTED;
  return hip_status(amq::launch_ternary(W, ld, (int)cols, (int)rows, T, planes, alpha,
                                        static_cast<hipStream_t>(stream)));
}

int amq_relative_mse(const float* W, int64_t rows, int64_t cols, int64_t ld, int k, const uint32_t* planes,
                     const float* alpha, double* row_err, double* row_norm, double* result, void* stream) {
  if (!W || !planes || !alpha || !row_err || !row_norm || !result) return AMQ_ERR_INVALID;
  if (!bits_ok(k) || rows <= 0 || cols <= 0 || ld < cols) return AMQ_ERR_INVALID;
  if (cols > (1 << 30) || rows > (1LL << 33)) return AMQ_ERR_UNSUPPORTED;
  return hip_status(amq::launch_relative_mse(W, rows, (int)cols, ld, k, planes, alpha, row_err, row_norm, result,
                                             static_cast<hipStream_t>(stream)));
}

int amq_embedding_lookup(const uint32_t* Ep, const float* alpha_e, int64_t vocab, int64_t n, int k,
                         const int64_t* ids, int64_t B, uint32_t* Xp, float* beta, void* stream) {
  if (!Ep || !alpha_e || !ids || !Xp || !beta) return AMQ_ERR_INVALID;
  if (!bits_ok(k) || vocab <= 0 || n <= 0 || B <= 0) return AMQ_ERR_INVALID;
  if (n > AMQ_MAX_QUANT_N || B > 0x7fffffffLL) return AMQ_ERR_UNSUPPORTED;
  amq::QuantArgs q{};
  q.mode = amq::kQuantFull;
  q.gather = amq::GatherSeg{Ep, alpha_e, vocab, reinterpret_cast<const long long*>(ids), (int)n, (int)B, Xp, beta};
  return hip_status(amq::launch_quantize(q, k, static_cast<hipStream_t>(stream)));
}

int amq_log_softmax(const float* Y, int64_t B, int64_t V, float* out, void* stream) {
  if (!Y || !out || B <= 0 || V <= 0) return AMQ_ERR_INVALID;
  if (B > 0x7fffffffLL || V > (1LL << 31)) return AMQ_ERR_UNSUPPORTED;
  return hip_status(amq::launch_log_softmax(Y, B, V, out, static_cast<hipStream_t>(stream)));
}

// Workspace of the output layer: the quantized h_t and the (max, sum of exponentials) pairs the
// product kernel leaves for the log-softmax.
struct SoftmaxWs {
  uint32_t* hp;
  float* beta;
  float* lse_part;
  int lse_cap;  // pairs per batch entry
  size_t total;
};
static SoftmaxWs carve_softmax(void* ws, int64_t V, int64_t H, int64_t B, int k_a) {
  SoftmaxWs w;
  char* base = static_cast<char*>(ws);
  size_t off = 0;
  w.hp = reinterpret_cast<uint32_t*>(base ? base + off : nullptr);
  off += up256(sizeof(uint32_t) * (size_t)k_a * B * amq_wpr(H));
  w.beta = reinterpret_cast<float*>(base ? base + off : nullptr);
  off += up256(sizeof(float) * (size_t)B * k_a);
  w.lse_part = reinterpret_cast<float*>(base ? base + off : nullptr);
  // pairs per batch entry: the small-batch kernel leaves one per wave (up to kLseMaxSlots), the
  // matrix-core kernels one per wave or workgroup of a batch tile's share of the grid (fewer the
  // more tiles there are); a launch that would need more leaves none and the stand-alone
  // log-softmax runs instead
  const int64_t cap = amq::bmv_supported((int)H, 0, k_a, B, amq::kEpiStore) ? amq::kLseMaxSlots : B <= 64 ? 4096 : 1024;
  w.lse_cap = (int)(V + 64 < cap ? V + 64 : cap);
  off += up256(sizeof(float) * 2 * (size_t)B * w.lse_cap);
  w.total = off;
  return w;
}

size_t amq_softmax_layer_workspace_bytes(int64_t V, int64_t H, int64_t B, int k_a) {
  if (V <= 0 || H <= 0 || B <= 0 || !bits_ok(k_a)) return 0;
  return carve_softmax(nullptr, V, H, B, k_a).total;
}

static int softmax_layer_launch(const uint32_t* Wsp, const float* alpha_s, int64_t V, int64_t H, int k_w,
                                const float* bias, const float* h, int64_t B, int k_a, int T, float* logprob,
                                const SoftmaxWs& w, hipStream_t s) {
  amq::QuantArgs q{};
  q.seg[0] = amq::QuantSeg{h, H, (int)H, (int)B, w.hp, w.beta};
  q.T = T;
  q.mode = amq::kQuantFull;
  int st = hip_status(amq::launch_quantize(q, k_a, s));
  if (st != AMQ_OK) return st;
  amq::GemmArgs g = gemm_args(Wsp, alpha_s, V, H, k_w, w.hp, w.beta, B, k_a, bias, 0, logprob);
  g.lse_part = B <= 65535 ? w.lse_part : nullptr;
  g.lse_cap = w.lse_cap;
  int slots = 0;
  st = run_product(g, s, &slots);
  if (st != AMQ_OK) return st;
  if (slots > 0) return hip_status(amq::launch_log_softmax_finish(logprob, B, V, w.lse_part, slots, logprob, s));
  return hip_status(amq::launch_log_softmax(logprob, B, V, logprob, s));
}

int amq_softmax_layer(const uint32_t* Wsp, const float* alpha_s, int64_t V, int64_t H, int k_w,
                      const float* bias, const float* h, int64_t B, int k_a, int T, float* logprob,
                      void* workspace, size_t workspace_bytes, void* stream) {
  if (!Wsp || !alpha_s || !h || !logprob || !workspace) return AMQ_ERR_INVALID;
  if (!bits_ok(k_w) || !bits_ok(k_a) || T < 0 || V <= 0 || H <= 0 || B <= 0) return AMQ_ERR_INVALID;
  if (!aligned(Wsp, 16) || !aligned(workspace, 256)) return AMQ_ERR_INVALID;
  if (workspace_bytes < carve_softmax(nullptr, V, H, B, k_a).total) return AMQ_ERR_INVALID;
  if (H > AMQ_MAX_QUANT_N || B > (1 << 24) || V > (1LL << 31)) return AMQ_ERR_UNSUPPORTED;
  SoftmaxWs w = carve_softmax(workspace, V, H, B, k_a);
  return softmax_layer_launch(Wsp, alpha_s, V, H, k_w, bias, h, B, k_a, T, logprob, w,
                              static_cast<hipStream_t>(stream));
}

// The recurrent half of a language-model step: lookup + on-line quantization (one launch), then the
// LSTM step; h and c are updated in place, hs_out (nullable) receives a copy of the new h.
static int lm_recurrent_launch(const uint32_t* Ep, const float* alpha_e, int64_t vocab, int64_t E,
                               const uint32_t* Wxp, const float* alpha_x, const uint32_t* Whp, const float* alpha_h,
                               int64_t H, int k_w, const float* bias, const int64_t* ids, float* h, float* c,
                               int64_t B, int k_a, int T, float* hs_out, const StepWs& w, hipStream_t s) {
  int st;
  // h_{t-1} quantized on line and x_t looked up in the quantized embedding, one launch
  amq::QuantArgs q{};
  q.seg[0] = amq::QuantSeg{h, H, (int)H, (int)B, w.hp, w.beta_h};
  q.T = T;
  q.mode = amq::kQuantFull;
  q.gather = amq::GatherSeg{Ep, alpha_e, vocab, reinterpret_cast<const long long*>(ids), (int)E, (int)B, w.xp,
                            w.beta_x};
  st = hip_status(amq::launch_quantize(q, k_a, s));
  if (st != AMQ_OK) return st;
  st = lstm_fused_launch(Wxp, alpha_x, Whp, alpha_h, E, H, k_w, bias, w.xp, w.beta_x, w.hp, w.beta_h, c, B, k_a,
                         h, c, hs_out, s);
  if (st < 0) {
    amq::GemmArgs gx = gemm_args(Wxp, alpha_x, 4 * H, E, k_w, w.xp, w.beta_x, B, k_a, bias, 0, w.pre0);
    st = run_product(gx, s);
    if (st != AMQ_OK) return st;
    amq::GemmArgs gh = gemm_args(Whp, alpha_h, 4 * H, H, k_w, w.hp, w.beta_h, B, k_a, nullptr, 1, w.pre0);
    st = run_product(gh, s);
    if (st != AMQ_OK) return st;
    st = hip_status(amq::launch_lstm_pointwise(w.pre0, c, h, c, hs_out, B, H, s));
  }
  return st;
}

// The launches of one language-model step on carved workspaces (arguments already validated).
static int lm_step_launch(const uint32_t* Ep, const float* alpha_e, int64_t vocab, int64_t E, const uint32_t* Wxp,
                          const float* alpha_x, const uint32_t* Whp, const float* alpha_h, int64_t H, int k_w,
                          const float* bias, const uint32_t* Wsp, const float* alpha_s, int64_t V, int k_ws,
                          const float* bias_s, const int64_t* ids, float* h, float* c, int64_t B, int k_a, int k_as,
                          int T, float* logprob, const StepWs& w, const SoftmaxWs& sw, hipStream_t s) {
  int st = lm_recurrent_launch(Ep, alpha_e, vocab, E, Wxp, alpha_x, Whp, alpha_h, H, k_w, bias, ids, h, c, B, k_a, T,
                               nullptr, w, s);
  if (st != AMQ_OK) return st;
  return softmax_layer_launch(Wsp, alpha_s, V, H, k_ws, bias_s, h, B, k_as, T, logprob, sw, s);
}

size_t amq_lm_workspace_bytes(int64_t E, int64_t H, int64_t V, int64_t B, int k_a, int k_as) {
  if (E <= 0 || H <= 0 || V <= 0 || B <= 0 || !bits_ok(k_a) || !bits_ok(k_as)) return 0;
  return carve(nullptr, E, H, B, k_a, 4, 1).total + carve_softmax(nullptr, V, H, B, k_as).total;
}

int amq_lm_step(const uint32_t* Ep, const float* alpha_e, int64_t vocab, int64_t E, const uint32_t* Wxp,
                const float* alpha_x, const uint32_t* Whp, const float* alpha_h, int64_t H, int k_w,
                const float* bias, const uint32_t* Wsp, const float* alpha_s, int64_t V, int k_ws,
                const float* bias_s, const int64_t* ids, float* h, float* c, int64_t B, int k_a, int k_as, int T,
                float* logprob, void* workspace, size_t workspace_bytes, void* stream) {
  if (!Ep || !alpha_e || !Wsp || !alpha_s || !ids || !c || !logprob) return AMQ_ERR_INVALID;
  if (vocab <= 0 || V <= 0 || !bits_ok(k_ws) || !bits_ok(k_as)) return AMQ_ERR_INVALID;
  const bool sizes_ok = E > 0 && H > 0 && B > 0 && bits_ok(k_a);
  const size_t need_step = sizes_ok ? carve(nullptr, E, H, B, k_a, 4, 1).total : 0;
  const size_t need = sizes_ok ? need_step + carve_softmax(nullptr, V, H, B, k_as).total : 0;
  int st = check_step(Wxp, alpha_x, Whp, alpha_h, E, H, k_w, ids, h, B, k_a, T, h, workspace, workspace_bytes,
                      need);
  if (st != AMQ_OK) return st;
  if (!aligned(Wsp, 16) || !aligned(Ep, 16)) return AMQ_ERR_INVALID;
  if (V > (1LL << 31)) return AMQ_ERR_UNSUPPORTED;
  hipStream_t s = static_cast<hipStream_t>(stream);
  StepWs w = carve(workspace, E, H, B, k_a, 4, 1);
  SoftmaxWs sw = carve_softmax(static_cast<char*>(workspace) + need_step, V, H, B, k_as);

  return lm_step_launch(Ep, alpha_e, vocab, E, Wxp, alpha_x, Whp, alpha_h, H, k_w, bias, Wsp, alpha_s, V, k_ws, bias_s,
                        ids, h, c, B, k_a, k_as, T, logprob, w, sw, s);
}

// Steps of a sequence whose hidden states go through the output layer together: as many as the
// batch-1 sequence kernel takes per launch, otherwise as many as give about 4096 rows.
static int64_t lm_piece_steps(int64_t B) {
  if (B == 1) return amq::kSeqGMaxSteps;
  return B >= 4096 ? 1 : 4096 / B;
}

// Workspace of amq_lm_sequence: that of a step, then every h_t of a piece of the sequence and the
// output layer's workspace for as many rows.
struct LmSeqWs {
  size_t step_bytes;
  float* hs;
  size_t soft_off;
  int soft_batch;
  // split recurrent step (batch > 1): the looked-up input codes of two consecutive steps, the x-side sums
  uint32_t* xq[2];
  float* xbeta[2];
  float* xsum;
  size_t total;
};
static LmSeqWs carve_lm_seq(void* ws, int64_t E, int64_t H, int64_t V, int64_t B, int k_a, int k_as) {
  LmSeqWs w;
  char* base = static_cast<char*>(ws);
  w.step_bytes = carve(nullptr, E, H, B, k_a, 4, 1).total;
  size_t off = w.step_bytes;
  w.hs = reinterpret_cast<float*>(base ? base + off : nullptr);
  w.soft_batch = (int)(lm_piece_steps(B) * B);
  off += up256(sizeof(float) * (size_t)w.soft_batch * H);
  w.soft_off = off;
  off += carve_softmax(nullptr, V, H, w.soft_batch, k_as).total;
  auto take = [&](size_t bytes) {
    char* p = base ? base + off : nullptr;
    off += up256(bytes);
    return p;
  };
  for (int i = 0; i < 2; ++i) {
    w.xq[i] = reinterpret_cast<uint32_t*>(take(sizeof(uint32_t) * (size_t)k_a * B * amq_wpr(E)));
    w.xbeta[i] = reinterpret_cast<float*>(take(sizeof(float) * (size_t)B * k_a));
  }
  w.xsum = reinterpret_cast<float*>(take(sizeof(float) * (size_t)B * H * 4));
  w.total = off;
  return w;
}

size_t amq_lm_sequence_workspace_bytes(int64_t E, int64_t H, int64_t V, int64_t B, int k_a, int k_as) {
  if (E <= 0 || H <= 0 || V <= 0 || B <= 0 || !bits_ok(k_a) || !bits_ok(k_as)) return 0;
  return carve_lm_seq(nullptr, E, H, V, B, k_a, k_as).total;
}

// Output side of a piece of a sequence: either log-probabilities of every word, or (scoring) the
// log-probability of one given word per row.
struct LmOutput {
  float* logprob;            // [steps][B][V], or null when scoring
  const int64_t* targets;    // [steps][B] when scoring
  float* target_logprob;     // [steps][B] when scoring
  float* tlogit;             // scoring scratch: the chosen logit of every row of a piece
  float* chunk_logprob;      // scoring scratch: log-probabilities of up to chunk_rows rows
  int64_t chunk_rows;
};

// Scoring pass of the output layer over `rows` hidden states: where the several-tiles product takes the
// shape, the logits are never written -- the kernel leaves the chosen logit of every row and the
// (max, sum) pairs, and a small kernel forms logit - log-sum-exp; otherwise chunks of rows go through the
// ordinary layer into a small buffer from which the chosen entries are gathered.
static int score_layer_launch(const uint32_t* Wsp, const float* alpha_s, int64_t V, int64_t H, int k_ws,
                              const float* bias_s, const float* hs, int64_t rows, int k_as, int T,
                              const int64_t* targets, float* out, char* soft_base, const LmOutput& o,
                              hipStream_t s) {
  const long long* tg = reinterpret_cast<const long long*>(targets);
  SoftmaxWs sw = carve_softmax(soft_base, V, H, rows, k_as);
  amq::BmvArgs b{};
  b.blk[0] = amq::BmvBlock{Wsp, alpha_s, sw.hp, sw.beta, (int)H};
  b.m = V;
  b.batch = (int)rows;
  b.bias0 = bias_s;
  b.lse_part = sw.lse_part;
  b.lse_cap = sw.lse_cap;
  b.tgt = tg;
  b.tgt_out = o.tlogit;
  b.groups = 1;
  if (!amq::bmv_supported((int)H, 0, k_as, rows, amq::kEpiStore) && amq::mfma4w_supported(b, k_ws, k_as)) {
    amq::QuantArgs q{};
    q.seg[0] = amq::QuantSeg{hs, H, (int)H, (int)rows, sw.hp, sw.beta};
    q.T = T;
    q.mode = amq::kQuantFull;
    int st = hip_status(amq::launch_quantize(q, k_as, s));
    if (st != AMQ_OK) return st;
    int slots = 0;
    st = hip_status(amq::launch_mfma4w(b, k_ws, k_as, s, &slots));
    if (st != AMQ_OK) return st;
    if (slots > 0)
      return hip_status(amq::launch_score_finish(o.tlogit, tg, rows, V, sw.lse_part, slots, out, s));
  }
  for (int64_t r0 = 0; r0 < rows; r0 += o.chunk_rows) {
    const int64_t n = rows - r0 < o.chunk_rows ? rows - r0 : o.chunk_rows;
    SoftmaxWs swc = carve_softmax(soft_base, V, H, n, k_as);
    int st = softmax_layer_launch(Wsp, alpha_s, V, H, k_ws, bias_s, hs + r0 * H, n, k_as, T, o.chunk_logprob, swc, s);
    if (st != AMQ_OK) return st;
    st = hip_status(amq::launch_gather_columns(o.chunk_logprob, n, V, tg + r0, out + r0, s));
    if (st != AMQ_OK) return st;
  }
  return AMQ_OK;
}

// Workspace of amq_lm_sequence_score: that of amq_lm_sequence, then one float per row of a piece and
// room for the log-probabilities of 64 rows.
struct LmScoreWs {
  float* tlogit;
  float* chunk_logprob;
  int64_t chunk_rows;
  size_t total;
};
static LmScoreWs carve_lm_score(void* ws, int64_t E, int64_t H, int64_t V, int64_t B, int k_a, int k_as) {
  LmScoreWs w;
  char* base = static_cast<char*>(ws);
  const LmSeqWs lw = carve_lm_seq(nullptr, E, H, V, B, k_a, k_as);
  size_t off = lw.total;
  w.tlogit = reinterpret_cast<float*>(base ? base + off : nullptr);
  off += up256(sizeof(float) * (size_t)lw.soft_batch);
  w.chunk_rows = lw.soft_batch < 64 ? lw.soft_batch : 64;
  w.chunk_logprob = reinterpret_cast<float*>(base ? base + off : nullptr);
  off += up256(sizeof(float) * (size_t)w.chunk_rows * V);
  w.total = off;
  return w;
}

static int lm_sequence_impl(const uint32_t* Ep, const float* alpha_e, int64_t vocab, int64_t E, const uint32_t* Wxp,
                            const float* alpha_x, const uint32_t* Whp, const float* alpha_h, int64_t H, int k_w,
                            const float* bias, const uint32_t* Wsp, const float* alpha_s, int64_t V, int k_ws,
                            const float* bias_s, const int64_t* ids, int64_t steps, float* h, float* c, int64_t B,
                            int k_a, int k_as, int T, LmOutput o, void* workspace, size_t workspace_bytes,
                            size_t need, void* stream) {
  int st = check_step(Wxp, alpha_x, Whp, alpha_h, E, H, k_w, ids, h, B, k_a, T, h, workspace, workspace_bytes,
                      need);
  if (st != AMQ_OK) return st;
  if (!aligned(Wsp, 16) || !aligned(Ep, 16)) return AMQ_ERR_INVALID;
  if (V > (1LL << 31) || steps >= (1 << 30)) return AMQ_ERR_UNSUPPORTED;
  hipStream_t s = static_cast<hipStream_t>(stream);
  LmSeqWs lw = carve_lm_seq(workspace, E, H, V, B, k_a, k_as);
  StepWs w = carve(workspace, E, H, B, k_a, 4, 1);
  char* soft_base = static_cast<char*>(workspace) + lw.soft_off;
  // every h_t of a piece of the sequence goes through the output layer together, as a batch of rows
  auto output_layer = [&](int64_t row0, int64_t rows) -> int {
    if (lw.soft_off + carve_softmax(nullptr, V, H, rows, k_as).total > workspace_bytes)
      return AMQ_ERR_INVALID;  // (cannot happen: fewer rows need less)
    if (o.logprob) {
      SoftmaxWs sw = carve_softmax(soft_base, V, H, rows, k_as);
      return softmax_layer_launch(Wsp, alpha_s, V, H, k_ws, bias_s, lw.hs, rows, k_as, T, o.logprob + row0 * V, sw, s);
    }
    return score_layer_launch(Wsp, alpha_s, V, H, k_ws, bias_s, lw.hs, rows, k_as, T, o.targets + row0,
                              o.target_logprob + row0, soft_base, o, s);
  };
  if (B == 1 && amq::lstm_seqg_supported(E, H, B, k_w, k_a) && grid_fits_device()) {
    // batch 1: per piece of at most kSeqGMaxSteps steps, look all inputs up (the table the sequence
    // kernel reads its input codes from), run the recurrence in one launch over the chip, then the
    // output layer
    for (int64_t t0 = 0; t0 < steps; t0 += amq::kSeqGMaxSteps) {
      const int n = (int)(steps - t0 < amq::kSeqGMaxSteps ? steps - t0 : amq::kSeqGMaxSteps);
      amq::QuantArgs q{};
      q.mode = amq::kQuantFull;
      q.gather = amq::GatherSeg{Ep, alpha_e, vocab, reinterpret_cast<const long long*>(ids + t0), (int)E, n, w.xq,
                                w.xbeta};
      st = hip_status(amq::launch_quantize(q, k_a, s));
      if (st != AMQ_OK) return st;
      amq::SeqGArgs g{Wxp, alpha_x, Whp, alpha_h, (int)E, (int)H, bias, nullptr, n, h, c, lw.hs, T, 0, w.sync, w.hbuf,
                      w.xq, w.xbeta, t0 == 0, 0};
      st = hip_status(amq::launch_lstm_seqg(g, k_w, k_a, s));
      if (st != AMQ_OK) return st;
      st = output_layer(t0, n);
      if (st != AMQ_OK) return st;
      // the output layer has just read hidden states that are incomplete if the recurrence gave up (now
      // or in an earlier piece of this call): its results for these steps become NaN
      st = hip_status(o.logprob ? amq::launch_seqg_poison(w.sync, o.logprob + t0 * V, (long long)n * V, s)
                                : amq::launch_seqg_poison(w.sync, o.target_logprob + t0, n, s));
      if (st != AMQ_OK) return st;
    }
    return AMQ_OK;
  }
  // The inputs are given (no step feeds on the outputs), so only the recurrence is serial: per
  // piece, the recurrent halves of its steps one after the other, every h_t kept, then one pass
  // of the output layer over all (step, batch entry) rows of the piece, which reads W_s once per
  // piece instead of once per step and runs its product at a shape the matrix cores fill.
  // The recurrent halves themselves: where the split step of amq_lstm_sequence applies, W_x x_t leaves the
  // chain here too -- the codes of x_t are rows of the quantized embedding, looked up one step ahead by
  // workgroups of the front launch (front launch of step t: quantize h_{t-1}, look up x_{t+1}, form the
  // x-side sums of step t; back launch: h-side sums + stored x-side sums + cell; the first step looks up
  // x_0 and x_1 and runs the whole-step kernel).  Same results as the per-step launches, bit for bit.
  const amq::BmvArgs probe = lstm_args(Wxp, alpha_x, Whp, alpha_h, E, H, bias, lw.xq[0], lw.xbeta[0], w.hp, w.beta_h, c,
                                       B, h, c, nullptr);
  const bool split = amq::step_split_supported(probe, k_w, k_a, amq::kEpiLstm);
  auto lookup = [&](int64_t u) {  // the inputs of step u into the code buffer of its parity
    return amq::GatherSeg{Ep, alpha_e, vocab, reinterpret_cast<const long long*>(ids + u * B), (int)E, (int)B,
                          lw.xq[u % 2], lw.xbeta[u % 2]};
  };
  auto split_step = [&](int64_t u, float* hs_out) -> int {
    amq::BmvArgs b = probe;
    b.blk[0].Xp = lw.xq[u % 2];
    b.blk[0].beta = lw.xbeta[u % 2];
    b.Y = lw.xsum;
    b.hs_out = hs_out;
    amq::QuantArgs q{}, q2{};
    q.seg[0] = amq::QuantSeg{h, H, (int)H, (int)B, w.hp, w.beta_h};
    q.T = q2.T = T;
    q.mode = q2.mode = amq::kQuantFull;
    int r;
    if (u == 0) {
      q.gather = lookup(0);
      if (steps > 1) q2.gather = lookup(1);
      r = hip_status(amq::launch_step_front(q, steps > 1 ? &q2 : nullptr, nullptr, k_w, k_a, amq::kEpiLstm, s));
      if (r != AMQ_OK) return r;
      return hip_status(amq::launch_mfma4_pair(b, k_w, k_a, amq::kEpiLstm, s));
    }
    if (u + 1 < steps) q.gather = lookup(u + 1);
    r = hip_status(amq::launch_step_front(q, nullptr, &b, k_w, k_a, amq::kEpiLstm, s));
    if (r != AMQ_OK) return r;
    return hip_status(amq::launch_step_back(b, k_w, k_a, amq::kEpiLstm, s));
  };
  const int64_t piece = lm_piece_steps(B);
  for (int64_t t0 = 0; t0 < steps; t0 += piece) {
    const int64_t n = steps - t0 < piece ? steps - t0 : piece;
    for (int64_t t = 0; t < n; ++t) {
      st = split ? split_step(t0 + t, lw.hs + t * B * H)
                 : lm_recurrent_launch(Ep, alpha_e, vocab, E, Wxp, alpha_x, Whp, alpha_h, H, k_w, bias,
                                       ids + (t0 + t) * B, h, c, B, k_a, T, lw.hs + t * B * H, w, s);
      if (st != AMQ_OK) return st;
    }
    st = output_layer(t0 * B, n * B);
    if (st != AMQ_OK) return st;
  }
  return AMQ_OK;
}

int amq_lm_sequence(const uint32_t* Ep, const float* alpha_e, int64_t vocab, int64_t E, const uint32_t* Wxp,
                    const float* alpha_x, const uint32_t* Whp, const float* alpha_h, int64_t H, int k_w,
                    const float* bias, const uint32_t* Wsp, const float* alpha_s, int64_t V, int k_ws,
                    const float* bias_s, const int64_t* ids, int64_t steps, float* h, float* c, int64_t B, int k_a,
                    int k_as, int T, float* logprob, void* workspace, size_t workspace_bytes, void* stream) {
  if (!Ep || !alpha_e || !Wsp || !alpha_s || !ids || !c || !logprob || steps <= 0) return AMQ_ERR_INVALID;
  if (vocab <= 0 || V <= 0 || !bits_ok(k_ws) || !bits_ok(k_as)) return AMQ_ERR_INVALID;
  const bool sizes_ok = E > 0 && H > 0 && B > 0 && bits_ok(k_a);
  const size_t need = sizes_ok ? carve_lm_seq(nullptr, E, H, V, B, k_a, k_as).total : 0;
  LmOutput o{logprob, nullptr, nullptr, nullptr, nullptr, 0};
  return lm_sequence_impl(Ep, alpha_e, vocab, E, Wxp, alpha_x, Whp, alpha_h, H, k_w, bias, Wsp, alpha_s, V, k_ws, bias_s,
                          ids, steps, h, c, B, k_a, k_as, T, o, workspace, workspace_bytes, need, stream);
}

size_t amq_lm_sequence_score_workspace_bytes(int64_t E, int64_t H, int64_t V, int64_t B, int k_a, int k_as) {
  if (E <= 0 || H <= 0 || V <= 0 || B <= 0 || !bits_ok(k_a) || !bits_ok(k_as)) return 0;
  return carve_lm_score(nullptr, E, H, V, B, k_a, k_as).total;
}

int amq_lm_sequence_score(const uint32_t* Ep, const float* alpha_e, int64_t vocab, int64_t E, const uint32_t* Wxp,
                          const float* alpha_x, const uint32_t* Whp, const float* alpha_h, int64_t H, int k_w,
                          const float* bias, const uint32_t* Wsp, const float* alpha_s, int64_t V, int k_ws,
                          const float* bias_s, const int64_t* ids, const int64_t* targets, int64_t steps, float* h,
                          float* c, int64_t B, int k_a, int k_as, int T, float* target_logprob, void* workspace,
                          size_t workspace_bytes, void* stream) {
  if (!Ep || !alpha_e || !Wsp || !alpha_s || !ids || !targets || !c || !target_logprob || steps <= 0)
    return AMQ_ERR_INVALID;
  if (vocab <= 0 || V <= 0 || !bits_ok(k_ws) || !bits_ok(k_as)) return AMQ_ERR_INVALID;
  const bool sizes_ok = E > 0 && H > 0 && B > 0 && bits_ok(k_a);
  if (sizes_ok && V > (1LL << 31)) return AMQ_ERR_UNSUPPORTED;
  const size_t need = sizes_ok ? carve_lm_score(nullptr, E, H, V, B, k_a, k_as).total : 0;
  LmOutput o{nullptr, targets, target_logprob, nullptr, nullptr, 0};
  if (sizes_ok && workspace) {
    const LmScoreWs sw = carve_lm_score(workspace, E, H, V, B, k_a, k_as);
    o.tlogit = sw.tlogit;
    o.chunk_logprob = sw.chunk_logprob;
    o.chunk_rows = sw.chunk_rows;
  }
  return lm_sequence_impl(Ep, alpha_e, vocab, E, Wxp, alpha_x, Whp, alpha_h, H, k_w, bias, Wsp, alpha_s, V, k_ws, bias_s,
                          ids, steps, h, c, B, k_a, k_as, T, o, workspace, workspace_bytes, need, stream);
}

}  // extern "C"
