// C ABI of libhot: argument checks, workspace layouts and the sequence of
// kernel launches behind each call declared in hot.h.  No device memory is
// allocated here; everything lives in caller-provided buffers.
#include <string.h>

#include <atomic>

#include "hot_host.h"

namespace hot {

namespace {

// Sign changes along row k of the +-1 Sylvester matrix, entry (k, j) = (-1)^popcount(k & j).
int row_sign_changes(int n, int k) {
  int changes = 0, prev = 0;
  for (int j = 0; j < n; ++j) {
    const int neg = __builtin_popcount((unsigned)(k & j)) & 1;
    if (j > 0 && neg != prev) ++changes;
    prev = neg;
  }
  return changes;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
// The workspace: its sub-regions (exchange slots, flags, operand rows) sit at multiples of 128
// and 256 bytes from its start and are accessed as 8- and 16-byte words.
bool aligned256(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 255u) == 0; }

}  // namespace

hot_status resolve_config(const hot_config* cfg, Config* out) {
  if (!cfg || !out) return HOT_ERR_ARG;
  const int n = cfg->block, r = cfg->keep;
  if (n != 16 && n != 32 && n != 64) return HOT_ERR_ARG;
  if (r < 1 || r > n) return HOT_ERR_ARG;
  if (cfg->gx_bits != 4 && cfg->gx_bits != 8) return HOT_ERR_ARG;
  if (cfg->gw_bits != 8 && cfg->gw_bits != 16) return HOT_ERR_ARG;
  if (cfg->rounding != HOT_ROUND_NEAREST_EVEN && cfg->rounding != HOT_ROUND_PSEUDO_STOCHASTIC)
    return HOT_ERR_ARG;
  if (!(cfg->lqs_threshold >= 0.0f)) return HOT_ERR_ARG;
  if (cfg->sample_tokens < 0) return HOT_ERR_ARG;
  out->n = n;
  out->r = r;
  out->gx_bits = cfg->gx_bits;
  out->gw_bits = cfg->gw_bits;
  out->rounding = cfg->rounding;
  out->lqs_threshold = cfg->lqs_threshold;
  out->sample_tokens = cfg->sample_tokens;
  if (cfg->replayable != 0 && cfg->replayable != 1) return HOT_ERR_ARG;
  out->replayable = cfg->replayable == 1;
  out->epoch = nullptr;
  out->lowpass_default = cfg->keep_idx == nullptr;
  for (int k = 0; k < 64; ++k) out->map.pos[k] = -1;
  for (int j = 0; j < r; ++j) {
    int k;
    if (cfg->keep_idx) {
      k = cfg->keep_idx[j];
      if (k < 0 || k >= n || out->map.pos[k] >= 0) return HOT_ERR_ARG;
    } else {
      // the row with exactly j sign changes (sequencies 0..n-1 each occur once)
      k = 0;
      while (k < n && row_sign_changes(n, k) != j) ++k;
    }
    out->keep[j] = k;
    out->map.pos[k] = (int8_t)j;
  }
  return HOT_OK;
}

RowTiling row_tiling(const Config& c, int64_t L) {
  RowTiling t{0, c.sample_tokens, 1};
  if (c.sample_tokens == 0) {
    if (L >= c.n && L % c.n == 0) t.nblk = L / c.n;
  } else if (L >= c.sample_tokens && L % c.sample_tokens == 0) {
    t.bps = (int)ceil_div(c.sample_tokens, c.n);
    t.nblk = L / c.sample_tokens * t.bps;
  }
  return t;
}

GxLayout gx_layout(const Config& c, int64_t L, int64_t O, int64_t I) {
  GxLayout g;
  g.pitch = round_up(O * c.gx_bits / 8, kPitchAlign);
  g.scalars = 0;
  g.sg = kWsPrefix;
  g.qg = g.sg + (size_t)round_up(L * 4, 256);
  g.qw = g.qg + (size_t)(L * g.pitch);
  g.partial = (size_t)round_up((int64_t)(g.qw + (size_t)(I * g.pitch)), 256);
  g.total = g.partial + gemm_scratch_bytes(L, I, g.pitch, c.gx_bits);
  return g;
}

GwLayout gw_layout(const Config& c, int64_t L, int64_t O, int64_t I) {
  GwLayout g;
  g.Lr = row_tiling(c, L).nblk * c.r;
  g.pitch = round_up(g.Lr * (c.gw_bits / 8), kPitchAlign);
  g.scalars = 0;
  g.qg = kWsPrefix;
  g.partial = g.qg + (size_t)round_up(O * g.pitch, 256);
  g.total = g.partial + gemm_scratch_bytes(O, I, g.pitch, c.gw_bits);
  return g;
}

SelLayout sel_layout(const Config&, int64_t L, int64_t) {
  SelLayout s;
  s.scalars = 0;
  s.rowmax = kWsPrefix;
  s.partial = s.rowmax + (size_t)round_up(L * 4, 256);
  s.total = s.partial + (size_t)L * 16;
  return s;
}

FusedLayout fused_layout(const Config& c, int64_t L, int64_t O, int64_t I) {
  FusedLayout f;
  f.gx = gx_layout(c, L, O, I);
  f.gw = gw_layout(c, L, O, I);
  f.s_gh = 16;
  f.rowpart = (size_t)round_up((int64_t)f.gx.total, 256);
  f.qgh = f.rowpart + (size_t)round_up(gy_fused_tiles_x(O) * L * 4, 256);
  f.partial = f.qgh + (size_t)round_up(O * f.gw.pitch, 256);   // shared by the two GEMMs
  const size_t sx = gemm_scratch_bytes(L, I, f.gx.pitch, c.gx_bits);
  const size_t sw = gemm_scratch_bytes(O, I, f.gw.pitch, c.gw_bits);
  f.total = f.partial + (sx > sw ? sx : sw);
  return f;
}

WeightLayout weight_layout(const Config& c, int64_t O, int64_t I) {
  WeightLayout w;
  w.pitch = round_up(O * c.gx_bits / 8, kPitchAlign);
  w.codes = kHeaderBytes;
  w.total = w.codes + (size_t)(I * w.pitch);
  return w;
}

ActLayout act_layout(const Config& c, int64_t L, int64_t I) {
  ActLayout a;
  a.Lr = row_tiling(c, L).nblk * c.r;
  a.pitch = round_up(a.Lr * (c.gw_bits / 8), kPitchAlign);
  a.codes = kHeaderBytes;
  a.total = a.codes + (size_t)(I * a.pitch);
  return a;
}

namespace {

bool gx_shape_ok(const Config& c, int64_t L, int64_t O, int64_t I) {
  return L >= 1 && I >= 1 && O >= c.n && O % c.n == 0 && L < (1ll << 31) && I < (1ll << 31) &&
         O <= (c.gx_bits == 4 ? kMaxK4 : kMaxK8);
}
// With the weight codes in a buffer of their own the workspace holds no weight rows: the
// GEMM scratch follows the g_y codes directly.
size_t gx_cached_partial(const GxLayout& g) { return (size_t)round_up((int64_t)g.qw, 256); }
size_t gx_cached_total(const GxLayout& g) { return gx_cached_partial(g) + (g.total - g.partial); }

bool tok_shape_ok(const Config& c, int64_t L, int64_t cols) {
  // the int32 bound on L' only binds integer accumulators; bfloat16 operands sum in fp32
  const int64_t nblk = row_tiling(c, L).nblk;
  return cols >= 1 && nblk >= 1 && cols < (1ll << 31) && L < (1ll << 31) &&
         (c.gw_bits == 16 || nblk * c.r <= kMaxK8);
}

// How hot_linear_backward produces the two views of g_y: 0 = by measurement (below),
// 1 = always the two separate paths, 2 = the shared passes whenever they exist, 3 = the
// separate paths with every kernel in a launch of its own (no combined weight / g_y launch).
std::atomic<int> g_backward_strategy{0};

bool shared_gy_passes_exist(const Config& c) {
  return gy_fused_supported(c) && c.gw_bits == 8 && c.sample_tokens == 0;
}

// The shared passes read g_y twice but are bound by the vector ALUs; the separate paths read
// it two or three times at HBM speed.  Measured on MI355X: the shared passes win for
// 16-row blocks once the HLA view no longer fits the single-pass kernel (its kept values,
// 4 bytes each, beyond about 80 MB of registers: three HBM passes otherwise); they lose for
// 32-row blocks (one more butterfly stage across lanes) and whenever the single pass applies.
bool shared_gy_passes(const Config& c, int64_t L, int64_t O) {
  if (!shared_gy_passes_exist(c)) return false;
  const int strategy = g_backward_strategy.load();
  if (strategy == 1 || strategy == 3) return false;
  if (strategy == 2) return true;
  const int64_t kept_bytes = row_tiling(c, L).nblk * c.r * O * 4;
  return c.n == 16 && kept_bytes > 80ll * 1000 * 1000;
}

KeepMap identity_map(int n) {
  KeepMap m;
  for (int k = 0; k < 64; ++k) m.pos[k] = k < n ? (int8_t)k : (int8_t)-1;
  return m;
}

#define HOT_TRY(expr)                         \
  do {                                        \
    if ((expr) != hipSuccess) return HOT_ERR_DEVICE; \
  } while (0)
// A launch bracketed by the optional stage timer.
#define HOT_STAGE(stage, expr)                \
  do {                                        \
    stage_begin(stage, s);                    \
    const hipError_t e_ = (expr);             \
    stage_end(stage, s);                      \
    if (e_ != hipSuccess) return HOT_ERR_DEVICE; \
  } while (0)

// A replayable call keeps a 64-bit epoch among the workspace's scalars and advances it before
// anything else; the kernels that exchange values through the workspace move their launch tags
// by it (effective_tag), so that a replay of a recorded call never repeats a tag.  The epoch
// needs no initial value: it only has to change.
__global__ void advance_epoch_kernel(unsigned long long* epoch) { *epoch = *epoch + 1ull; }

hipError_t begin_call(Config& c, void* ws, hipStream_t s) {
  c.epoch = nullptr;
  if (!c.replayable) return hipSuccess;
  unsigned long long* e = (unsigned long long*)((uint8_t*)ws + kEpochOffset);
  advance_epoch_kernel<<<dim3(1), dim3(1), 0, s>>>(e);
  c.epoch = e;
  return hipGetLastError();
}

}  // namespace
}  // namespace hot

using namespace hot;

extern "C" {

void hot_default_config(hot_config* cfg) {
  if (!cfg) return;
  cfg->block = 16;
  cfg->keep = 8;
  cfg->keep_idx = nullptr;
  cfg->gx_bits = 4;
  cfg->gw_bits = 8;
  cfg->rounding = HOT_ROUND_PSEUDO_STOCHASTIC;
  cfg->lqs_threshold = 0.5f;
  cfg->sample_tokens = 0;
  cfg->replayable = 0;
}

const char* hot_status_string(hot_status s) {
  switch (s) {
    case HOT_OK: return "ok";
    case HOT_ERR_ARG: return "invalid argument";
    case HOT_ERR_SHAPE: return "unsupported shape";
    case HOT_ERR_WORKSPACE: return "workspace too small";
    case HOT_ERR_DEVICE: return "HIP runtime error";
    case HOT_ERR_UNIMPLEMENTED: return "not implemented";
    case HOT_ERR_SCRATCH_LIMIT: return "shape needs more scratch than the library's built-in buffer holds";
  }
  return "unknown status";
}

size_t hot_act_buffer_bytes(const hot_config* cfg, int64_t L, int64_t I) {
  Config c;
  if (resolve_config(cfg, &c) != HOT_OK || !tok_shape_ok(c, L, I)) return 0;
  return act_layout(c, L, I).total;
}

size_t hot_workspace_bytes(const hot_config* cfg, int64_t L, int64_t O, int64_t I) {
  Config c;
  if (resolve_config(cfg, &c) != HOT_OK) return 0;
  if (L < 1 || O < 1 || I < 1) return 0;
  size_t need = kWsPrefix;
  if (gx_shape_ok(c, L, O, I)) {
    const size_t a = gx_layout(c, L, O, I).total, b = sel_layout(c, L, O).total;
    need = a > need ? a : need;
    need = b > need ? b : need;
  }
  if (tok_shape_ok(c, L, O) && tok_shape_ok(c, L, I)) {
    const size_t a = gw_layout(c, L, O, I).total;
    need = a > need ? a : need;
    if (gx_shape_ok(c, L, O, I)) {   // hot_linear_backward keeps both operand sets at once
      const size_t b = fused_layout(c, L, O, I).total;
      need = b > need ? b : need;
    }
  }
  return need;
}

hot_status hot_compress_activation(const hot_config* cfg, const float* x, int64_t L, int64_t I,
                                   void* act_buf, void* ws, size_t ws_bytes, void* stream) {
  Config c;
  hot_status st = resolve_config(cfg, &c);
  if (st != HOT_OK) return st;
  if (!x || !act_buf || !ws || !aligned16(x) || !aligned16(act_buf) || !aligned256(ws)) return HOT_ERR_ARG;
  if (!tok_shape_ok(c, L, I)) return HOT_ERR_SHAPE;
  if (ws_bytes < (size_t)kWsPrefix) return HOT_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  const ActLayout a = act_layout(c, L, I);
  uint8_t* base = (uint8_t*)act_buf;
  float* partials = (float*)((uint8_t*)ws + kHeaderBytes);
  HOT_TRY(begin_call(c, ws, s));
  if (c.gw_bits == 16) {
    HOT_TRY(launch_col_bf16(x, row_tiling(c, L), I, c, base + a.codes, a.pitch, (float*)base, s, kStActQuant));
    return HOT_OK;
  }
  HOT_TRY(launch_col_quant(x, row_tiling(c, L), I, c, c.r, c.map, false, c.gw_bits, base + a.codes, a.pitch,
                           (float*)base, partials, s, kStActAbsmax, kStActQuant));
  return HOT_OK;
}

size_t hot_weight_buffer_bytes(const hot_config* cfg, int64_t O, int64_t I) {
  Config c;
  if (resolve_config(cfg, &c) != HOT_OK || !gx_shape_ok(c, 1, O, I)) return 0;
  return weight_layout(c, O, I).total;
}

size_t hot_gx_cached_workspace_bytes(const hot_config* cfg, int64_t L, int64_t O, int64_t I) {
  Config c;
  if (resolve_config(cfg, &c) != HOT_OK || !gx_shape_ok(c, L, O, I)) return 0;
  return gx_cached_total(gx_layout(c, L, O, I));
}

hot_status hot_quantize_weight(const hot_config* cfg, const float* w, int64_t O, int64_t I,
                               void* wq_buf, void* ws, size_t ws_bytes, void* stream) {
  Config c;
  hot_status st = resolve_config(cfg, &c);
  if (st != HOT_OK) return st;
  if (!w || !wq_buf || !ws || !aligned16(w) || !aligned16(wq_buf) || !aligned256(ws)) return HOT_ERR_ARG;
  if (!gx_shape_ok(c, 1, O, I)) return HOT_ERR_SHAPE;
  if (ws_bytes < (size_t)kWsPrefix) return HOT_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  const WeightLayout wl = weight_layout(c, O, I);
  uint8_t* base = (uint8_t*)wq_buf;
  float* partials = (float*)((uint8_t*)ws + kHeaderBytes);
  HOT_TRY(begin_call(c, ws, s));
  HOT_TRY(launch_col_quant(w, RowTiling{O / c.n, 0, 1}, I, c, c.n, identity_map(c.n), true, c.gx_bits, base + wl.codes,
                           wl.pitch, (float*)base, partials, s, kStWAbsmax, kStWQuant));
  return HOT_OK;
}

namespace {

// One GEMM on K-contiguous operands of `pitch` bytes, planned for its shape, with the
// scratch region at base + partial_off and the flag slots of the workspace prefix.
hipError_t gemm(const Config& c, const uint8_t* A, const uint8_t* B, int64_t M, int64_t N, int64_t pitch,
                int bits, uint8_t* base, size_t partial_off, int32_t* out_i32, float* out_f32,
                const float* row_scale, int row_stride, const float* col_scale, int n, hipStream_t s,
                int stage = -1) {
  return launch_igemm(A, B, M, N, pitch, pitch, bits, plan_gemm(M, N, pitch, bits, true),
                      (int32_t*)(base + partial_off), (unsigned long long*)(base + kGemmFlagsOffset),
                      out_i32, out_f32, row_scale, row_stride, col_scale, n, s, stage, c.epoch);
}



// g_x path, first half: the rotated, quantised g_y operand (codes at g.qg, scales at g.sg).
hot_status gx_rows(const Config& c, const float* g_y, int64_t L, int64_t O, hot_quantizer gy_quantizer,
                   uint8_t* base, const GxLayout& g, hipStream_t s) {
  float* part_g = (float*)(base + kHeaderBytes + kPartialBytes);
  float* s_g = (float*)(base + g.sg);
  uint8_t* qg = base + g.qg;
  int npart = 0;
  if (gy_quantizer == HOT_Q_PER_TOKEN) {
    HOT_STAGE(kStGyRowQuant, launch_row_quant(g_y, L, O, c.n, c.gx_bits, c.rounding, 0, qg, g.pitch, s_g, part_g, &npart, s));
  } else {
    HOT_STAGE(kStGyRowAbsmax, launch_row_quant(g_y, L, O, c.n, c.gx_bits, c.rounding, 1, qg, g.pitch, s_g, part_g, &npart, s));
    HOT_STAGE(kStGyRowQuant2, launch_row_quant(g_y, L, O, c.n, c.gx_bits, c.rounding, 2, qg, g.pitch, s_g, part_g, &npart, s));
  }
  return HOT_OK;
}

// g_x path, both operands from fp32 inputs: Q(H.w) as [I x O] code rows with its scale at
// g.scalars, and gx_rows; in one launch where that exists, else one after the other.
hot_status gx_operands(const Config& c, const float* g_y, const float* w, int64_t L, int64_t O, int64_t I,
                       hot_quantizer gy_quantizer, uint8_t* base, const GxLayout& g, hipStream_t s) {
  float* s_w = (float*)(base + g.scalars);
  float* part_w = (float*)(base + kHeaderBytes);
  uint8_t* qw = base + g.qw;
  bool both = false;
  if (gy_quantizer == HOT_Q_PER_TOKEN && g_backward_strategy.load() != 3)
    HOT_TRY(launch_w_and_rows(w, O, I, c, qw, g.pitch, s_w, part_w, g_y, L, base + g.qg,
                              (float*)(base + g.sg), s, kStWGyRow, &both));
  if (both) return HOT_OK;
  HOT_TRY(launch_col_quant(w, RowTiling{O / c.n, 0, 1}, I, c, c.n, identity_map(c.n), true, c.gx_bits, qw, g.pitch, s_w,
                           part_w, s, kStWAbsmax, kStWQuant));
  return gx_rows(c, g_y, L, O, gy_quantizer, base, g, s);
}

// g_x path, second half: multiply the operand at g.qg with quantised weights, dequantise.
hot_status gx_gemm(const Config& c, const uint8_t* qw, const float* s_w, int64_t L, int64_t I,
                   hot_quantizer gy_quantizer, float* g_x, uint8_t* base, const GxLayout& g,
                   size_t partial_off, hipStream_t s) {
  HOT_TRY(gemm(c, base + g.qg, qw, L, I, g.pitch, c.gx_bits, base, partial_off, nullptr, g_x,
               (const float*)(base + g.sg), gy_quantizer == HOT_Q_PER_TOKEN ? 1 : 0, s_w, c.n, s, kStGxGemm));
  return HOT_OK;
}

// HLA(g_y) along L as [O x L'] code rows at `qg` with its scale at `s_g` (INT8: one scale;
// bfloat16: no scale, 1 is stored), then the GEMM with the stored activation and dequantise.
hot_status gw_operand(const Config& c, const float* g_y, int64_t L, int64_t O, uint8_t* qg, int64_t pitch,
                      float* s_g, float* slots, hipStream_t s) {
  if (c.gw_bits == 16)
    HOT_TRY(launch_col_bf16(g_y, row_tiling(c, L), O, c, qg, pitch, s_g, s, kStGyTQuant));
  else
    HOT_TRY(launch_col_quant(g_y, row_tiling(c, L), O, c, c.r, c.map, false, c.gw_bits, qg, pitch, s_g, slots, s,
                             kStGyTAbsmax, kStGyTQuant));
  return HOT_OK;
}


}  // namespace

namespace {

// Checks shared by the two forms of the g_x call (everything but the scratch).
hot_status gx_check(const hot_config* cfg, const float* g_y, const float* w, int64_t L, int64_t O,
                    int64_t I, hot_quantizer gy_quantizer, const float* g_x, Config* c) {
  hot_status st = resolve_config(cfg, c);
  if (st != HOT_OK) return st;
  if (!g_y || !w || !g_x || !aligned16(g_y) || !aligned16(w) || !aligned16(g_x)) return HOT_ERR_ARG;
  if (gy_quantizer != HOT_Q_PER_TENSOR && gy_quantizer != HOT_Q_PER_TOKEN) return HOT_ERR_ARG;
  if (!gx_shape_ok(*c, L, O, I)) return HOT_ERR_SHAPE;
  return HOT_OK;
}

hot_status gx_run(const Config& c, const float* g_y, const float* w, int64_t L, int64_t O, int64_t I,
                  hot_quantizer gy_quantizer, float* g_x, uint8_t* base, const GxLayout& g, hipStream_t s) {
  hot_status st = gx_operands(c, g_y, w, L, O, I, gy_quantizer, base, g, s);
  if (st != HOT_OK) return st;
  return gx_gemm(c, base + g.qw, (const float*)(base + g.scalars), L, I, gy_quantizer, g_x, base, g, g.partial, s);
}

}  // namespace

hot_status hot_linear_backward_gx(const hot_config* cfg, const float* g_y, const float* w,
                                  int64_t L, int64_t O, int64_t I, hot_quantizer gy_quantizer,
                                  float* g_x, void* ws, size_t ws_bytes, void* stream) {
  Config c;
  hot_status st = gx_check(cfg, g_y, w, L, O, I, gy_quantizer, g_x, &c);
  if (st != HOT_OK) return st;
  if (!ws || !aligned256(ws)) return HOT_ERR_ARG;
  const GxLayout g = gx_layout(c, L, O, I);
  if (ws_bytes < g.total) return HOT_ERR_WORKSPACE;
  HOT_TRY(begin_call(c, ws, (hipStream_t)stream));
  return gx_run(c, g_y, w, L, O, I, gy_quantizer, g_x, (uint8_t*)ws, g, (hipStream_t)stream);
}

// ---- the g_x call for callers that cannot allocate ---------------------------------------
//
// The workspace of hot_linear_backward_gx (scalars, exchange slots, split-K flags, both packed
// operands, split-K images) lives in this array instead of a caller's buffer.  Every GPU the
// library runs on holds its own copy from the moment the code object is loaded until the
// process ends.  In host code the array's name is only a handle for hipGetSymbolAddress: the
// device address it returns (one per device) is what kernels, copies and fills are given.
static __device__ __attribute__((used)) __align__(256) unsigned char scratch[HOT_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_addr[kMaxDevices];

// Device address of `scratch` on the current device, looked up once per device.
hot_status scratch_of_current_device(uint8_t** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return HOT_ERR_DEVICE;
  void* p = g_scratch_addr[dev].load(std::memory_order_acquire);
  if (!p) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return HOT_ERR_DEVICE;
    if ((reinterpret_cast<uintptr_t>(p) & 255u) != 0) return HOT_ERR_DEVICE;
    g_scratch_addr[dev].store(p, std::memory_order_release);   // two threads racing here store the same address
  }
  *out = (uint8_t*)p;
  return HOT_OK;
}

}  // namespace

hot_status hot_linear_backward_gx_noalloc(const hot_config* cfg, const float* g_y, const float* w,
                                          int64_t L, int64_t O, int64_t I, hot_quantizer gy_quantizer,
                                          float* g_x, void* stream) {
  Config c;
  hot_status st = gx_check(cfg, g_y, w, L, O, I, gy_quantizer, g_x, &c);
  if (st != HOT_OK) return st;
  const GxLayout g = gx_layout(c, L, O, I);
  if (g.total > (size_t)HOT_NOALLOC_SCRATCH_BYTES) return HOT_ERR_SCRATCH_LIMIT;
  uint8_t* base = nullptr;
  st = scratch_of_current_device(&base);
  if (st != HOT_OK) return st;
  // Nothing in the scratch has to start at zero: exchange slots and split-K flags are told
  // from an earlier call's by a per-launch tag, everything else is written before it is read.
  HOT_TRY(begin_call(c, base, (hipStream_t)stream));
  return gx_run(c, g_y, w, L, O, I, gy_quantizer, g_x, base, g, (hipStream_t)stream);
}

hot_status hot_linear_backward_gx_cached(const hot_config* cfg, const float* g_y,
                                         const void* wq_buf, int64_t L, int64_t O, int64_t I,
                                         hot_quantizer gy_quantizer, float* g_x, void* ws,
                                         size_t ws_bytes, void* stream) {
  Config c;
  hot_status st = resolve_config(cfg, &c);
  if (st != HOT_OK) return st;
  if (!g_y || !wq_buf || !g_x || !ws || !aligned16(g_y) || !aligned16(wq_buf) || !aligned16(g_x) ||
      !aligned256(ws))
    return HOT_ERR_ARG;
  if (gy_quantizer != HOT_Q_PER_TENSOR && gy_quantizer != HOT_Q_PER_TOKEN) return HOT_ERR_ARG;
  if (!gx_shape_ok(c, L, O, I)) return HOT_ERR_SHAPE;
  const GxLayout g = gx_layout(c, L, O, I);
  if (ws_bytes < gx_cached_total(g)) return HOT_ERR_WORKSPACE;
  const WeightLayout wl = weight_layout(c, O, I);
  const uint8_t* wb = (const uint8_t*)wq_buf;
  HOT_TRY(begin_call(c, ws, (hipStream_t)stream));
  st = gx_rows(c, g_y, L, O, gy_quantizer, (uint8_t*)ws, g, (hipStream_t)stream);
  if (st != HOT_OK) return st;
  return gx_gemm(c, wb + wl.codes, (const float*)wb, L, I, gy_quantizer, g_x, (uint8_t*)ws, g,
                 gx_cached_partial(g), (hipStream_t)stream);
}

hot_status hot_linear_backward_gw(const hot_config* cfg, const float* g_y, const void* act_buf,
                                  int64_t L, int64_t O, int64_t I, float* g_w, void* ws,
                                  size_t ws_bytes, void* stream) {
  Config c;
  hot_status st = resolve_config(cfg, &c);
  if (st != HOT_OK) return st;
  if (!g_y || !act_buf || !g_w || !ws || !aligned16(g_y) || !aligned16(act_buf) || !aligned16(g_w) ||
      !aligned256(ws))
    return HOT_ERR_ARG;
  if (!tok_shape_ok(c, L, O) || !tok_shape_ok(c, L, I)) return HOT_ERR_SHAPE;
  const GwLayout g = gw_layout(c, L, O, I);
  if (ws_bytes < g.total) return HOT_ERR_WORKSPACE;
  const ActLayout a = act_layout(c, L, I);
  hipStream_t s = (hipStream_t)stream;
  uint8_t* base = (uint8_t*)ws;
  float* s_g = (float*)(base + g.scalars);
  float* part_g = (float*)(base + kHeaderBytes);
  uint8_t* qg = base + g.qg;
  const uint8_t* abase = (const uint8_t*)act_buf;

  HOT_TRY(begin_call(c, ws, s));
  st = gw_operand(c, g_y, L, O, qg, g.pitch, s_g, part_g, s);
  if (st != HOT_OK) return st;
  HOT_TRY(gemm(c, qg, abase + a.codes, O, I, g.pitch, c.gw_bits, base, g.partial, nullptr, g_w, s_g, 0,
               (const float*)abase, c.n, s, kStGwGemm));
  return HOT_OK;
}

hot_status hot_linear_backward(const hot_config* cfg, const float* g_y, const float* w,
                               const void* act_buf, int64_t L, int64_t O, int64_t I,
                               hot_quantizer gy_quantizer, float* g_x, float* g_w, void* ws,
                               size_t ws_bytes, void* stream) {
  Config c;
  hot_status st = resolve_config(cfg, &c);
  if (st != HOT_OK) return st;
  if (!g_y || !w || !act_buf || !g_x || !g_w || !ws || !aligned16(g_y) || !aligned16(w) ||
      !aligned16(act_buf) || !aligned16(g_x) || !aligned16(g_w) || !aligned256(ws))
    return HOT_ERR_ARG;
  if (gy_quantizer != HOT_Q_PER_TOKEN && gy_quantizer != HOT_Q_PER_TENSOR) return HOT_ERR_ARG;
  if (!gx_shape_ok(c, L, O, I) || !tok_shape_ok(c, L, O) || !tok_shape_ok(c, L, I)) return HOT_ERR_SHAPE;
  const FusedLayout f = fused_layout(c, L, O, I);
  const ActLayout a = act_layout(c, L, I);
  hipStream_t s = (hipStream_t)stream;
  uint8_t* base = (uint8_t*)ws;
  if (ws_bytes < f.total) return HOT_ERR_WORKSPACE;
  HOT_TRY(begin_call(c, ws, s));
  if (!shared_gy_passes(c, L, O)) {
    // The two separate paths, with both operand transforms ahead of both GEMMs (the workspace
    // holds the two operand sets side by side): the second reader of g_y follows the first
    // while part of the tensor is still in the memory-side cache, and no bandwidth-bound
    // kernel starts right behind the g_x GEMM, whose last 256 MB of output are then still on
    // their way from that cache to HBM (a streaming read behind a 1 GB write runs at 73 % of
    // its rate); the g_w GEMM, which moves few bytes, runs there instead.
    st = gx_operands(c, g_y, w, L, O, I, gy_quantizer, base, f.gx, s);
    if (st != HOT_OK) return st;
    st = gw_operand(c, g_y, L, O, base + f.qgh, f.gw.pitch, (float*)(base + f.s_gh), (float*)(base + kHeaderBytes), s);
    if (st != HOT_OK) return st;
    st = gx_gemm(c, base + f.gx.qw, (const float*)(base + f.gx.scalars), L, I, gy_quantizer, g_x, base, f.gx,
                 f.partial, s);
    if (st != HOT_OK) return st;
    HOT_TRY(gemm(c, base + f.qgh, (const uint8_t*)act_buf + a.codes, O, I, f.gw.pitch, c.gw_bits, base, f.partial,
                 nullptr, g_w, (const float*)(base + f.s_gh), 0, (const float*)act_buf, c.n, s, kStGwGemm));
    return HOT_OK;
  }
  float* s_w = (float*)(base + f.gx.scalars);
  float* s_gh = (float*)(base + f.s_gh);
  float* part_a = (float*)(base + kHeaderBytes);
  float* part_b = (float*)(base + kHeaderBytes + kPartialBytes);
  float* s_g = (float*)(base + f.gx.sg);
  uint8_t* qg = base + f.gx.qg;
  uint8_t* qw = base + f.gx.qw;
  uint8_t* qgh = base + f.qgh;
  const uint8_t* abase = (const uint8_t*)act_buf;
  const bool per_token = gy_quantizer == HOT_Q_PER_TOKEN;

  HOT_TRY(launch_col_quant(w, RowTiling{O / c.n, 0, 1}, I, c, c.n, identity_map(c.n), true, c.gx_bits, qw, f.gx.pitch, s_w,
                           part_a, s, kStWAbsmax, kStWQuant));
  HOT_TRY(launch_gy_fused(g_y, L, O, c, per_token, qg, f.gx.pitch, s_g, qgh, f.gw.pitch, s_gh, part_a,
                          part_b, (float*)(base + f.rowpart), s, kStGyFusedAbsmax, kStGyFusedQuant));
  HOT_TRY(gemm(c, qg, qw, L, I, f.gx.pitch, c.gx_bits, base, f.partial, nullptr, g_x, s_g,
               per_token ? 1 : 0, s_w, c.n, s, kStGxGemm));
  HOT_TRY(gemm(c, qgh, abase + a.codes, O, I, f.gw.pitch, c.gw_bits, base, f.partial, nullptr, g_w, s_gh,
               0, (const float*)abase, c.n, s, kStGwGemm));
  return HOT_OK;
}

hot_status hot_select_quantizer(const hot_config* cfg, const float* g_y, int64_t L, int64_t O,
                                hot_quantizer* choice, double* mse_token, double* mse_tensor,
                                void* ws, size_t ws_bytes, void* stream) {
  Config c;
  hot_status st = resolve_config(cfg, &c);
  if (st != HOT_OK) return st;
  if (!g_y || !choice || !ws || !aligned16(g_y) || !aligned256(ws)) return HOT_ERR_ARG;
  if (!gx_shape_ok(c, L, O, 1)) return HOT_ERR_SHAPE;
  const SelLayout l = sel_layout(c, L, O);
  if (ws_bytes < l.total) return HOT_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  uint8_t* base = (uint8_t*)ws;
  float* part = (float*)(base + kHeaderBytes);
  double* result = (double*)(base + l.scalars + 64);
  float* rowmax = (float*)(base + l.rowmax);
  double* partial = (double*)(base + l.partial);

  int npart = 0;
  HOT_TRY(launch_row_quant(g_y, L, O, c.n, c.gx_bits, c.rounding, 3, nullptr, 0, rowmax, part, &npart, s));
  HOT_TRY(launch_quant_error(g_y, L, O, c.n, c.gx_bits, c.rounding, rowmax, part, npart, partial, result, s));
  double host[2] = {0.0, 0.0};
  HOT_TRY(hipMemcpyAsync(host, result, sizeof(host), hipMemcpyDeviceToHost, s));
  HOT_TRY(hipStreamSynchronize(s));
  // errors were summed on the rotated tensor; H_u / sqrt(n) is orthonormal, hence the 1/n
  const double denom = (double)c.n * (double)L * (double)O;
  const double m_tok = host[0] / denom, m_ten = host[1] / denom;
  if (mse_token) *mse_token = m_tok;
  if (mse_tensor) *mse_tensor = m_ten;
  *choice = (m_ten > 0.0 && (m_ten - m_tok) >= (double)c.lqs_threshold * m_ten) ? HOT_Q_PER_TOKEN
                                                                               : HOT_Q_PER_TENSOR;
  return HOT_OK;
}

hot_status hot_lowpass_l1_rows(int32_t block, int32_t keep, int32_t* keep_idx) {
  const int n = block, r = keep;
  if (n != 16 && n != 32 && n != 64) return HOT_ERR_ARG;
  if (r < 1 || r > n || !keep_idx) return HOT_ERR_ARG;
  // H_n = H_gh (x) H_gw: natural row k = a * gw + b is the product of row a of H_gh, running
  // down the token grid, and row b of H_gw, running along it; its 2-D sequency is the pair of
  // their 1-D sequencies.
  const int gw = n == 16 ? 4 : 8, gh = n / gw;
  int key[64];
  for (int k = 0; k < n; ++k) {
    const int sv = row_sign_changes(gh, k / gw), sh = row_sign_changes(gw, k % gw);
    key[k] = ((sv + sh) * 64 + (sv > sh ? sv : sh)) * 64 + sv;
  }
  bool taken[64] = {false};
  for (int j = 0; j < r; ++j) {
    int best = -1;
    for (int k = 0; k < n; ++k)
      if (!taken[k] && (best < 0 || key[k] < key[best])) best = k;
    taken[best] = true;
    keep_idx[j] = best;
  }
  return HOT_OK;
}

hot_status hot_debug_unpack_activation(const hot_config* cfg, const void* act_buf, int64_t L,
                                       int64_t I, int8_t* codes, float* scale, void* stream) {
  Config c;
  hot_status st = resolve_config(cfg, &c);
  if (st != HOT_OK) return st;
  if (!act_buf) return HOT_ERR_ARG;
  if (!tok_shape_ok(c, L, I)) return HOT_ERR_SHAPE;
  const ActLayout a = act_layout(c, L, I);
  hipStream_t s = (hipStream_t)stream;
  const uint8_t* base = (const uint8_t*)act_buf;
  if (codes) HOT_TRY(launch_unpack(base + a.codes, I, a.Lr, a.pitch, c.gw_bits, 1, codes, s));
  if (scale) HOT_TRY(hipMemcpyAsync(scale, base, 4, hipMemcpyDeviceToDevice, s));
  return HOT_OK;
}

hot_status hot_debug_set_backward_strategy(int strategy) {
  if (strategy < 0 || strategy > 3) return HOT_ERR_ARG;
  g_backward_strategy.store(strategy);
  return HOT_OK;
}

hot_status hot_debug_set_exchange_wait_us(int us) {
  set_exchange_wait_us(us);
  set_gemm_wait_us(us);
  return HOT_OK;
}

hot_status hot_debug_set_gemm_mode(int mode) {
  if (mode < 0 || (mode > 8 && mode < 10) || mode > 13) return HOT_ERR_ARG;
  set_gemm_mode(mode);
  return HOT_OK;
}

hot_status hot_debug_unpack_weight(const hot_config* cfg, const void* wq_buf, int64_t O, int64_t I,
                                   int8_t* codes, float* scale, void* stream) {
  Config c;
  hot_status st = resolve_config(cfg, &c);
  if (st != HOT_OK) return st;
  if (!wq_buf) return HOT_ERR_ARG;
  if (!gx_shape_ok(c, 1, O, I)) return HOT_ERR_SHAPE;
  const WeightLayout wl = weight_layout(c, O, I);
  hipStream_t s = (hipStream_t)stream;
  const uint8_t* base = (const uint8_t*)wq_buf;
  if (codes) HOT_TRY(launch_unpack(base + wl.codes, I, O, wl.pitch, c.gx_bits, 1, codes, s));
  if (scale) HOT_TRY(hipMemcpyAsync(scale, base, 4, hipMemcpyDeviceToDevice, s));
  return HOT_OK;
}

hot_status hot_debug_gx_operands(const hot_config* cfg, void* ws, int64_t L, int64_t O,
                                 int64_t I, hot_quantizer gy_quantizer, int8_t* gy_codes,
                                 float* gy_scales, int8_t* w_codes, float* w_scale, int32_t* acc,
                                 void* stream) {
  Config c;
  hot_status st = resolve_config(cfg, &c);
  if (st != HOT_OK) return st;
  if (!ws) return HOT_ERR_ARG;
  if (!gx_shape_ok(c, L, O, I)) return HOT_ERR_SHAPE;
  const GxLayout g = gx_layout(c, L, O, I);
  hipStream_t s = (hipStream_t)stream;
  uint8_t* base = (uint8_t*)ws;
  if (gy_codes) HOT_TRY(launch_unpack(base + g.qg, L, O, g.pitch, c.gx_bits, 0, gy_codes, s));
  if (w_codes) HOT_TRY(launch_unpack(base + g.qw, I, O, g.pitch, c.gx_bits, 1, w_codes, s));
  if (gy_scales)
    HOT_TRY(hipMemcpyAsync(gy_scales, base + g.sg, gy_quantizer == HOT_Q_PER_TOKEN ? L * 4 : 4,
                           hipMemcpyDeviceToDevice, s));
  if (w_scale) HOT_TRY(hipMemcpyAsync(w_scale, base + g.scalars, 4, hipMemcpyDeviceToDevice, s));
  if (acc)
    HOT_TRY(gemm(c, base + g.qg, base + g.qw, L, I, g.pitch, c.gx_bits, base, g.partial, acc, nullptr,
                 nullptr, 0, nullptr, c.n, s));
  return HOT_OK;
}

hot_status hot_debug_gw_operands(const hot_config* cfg, void* ws, const void* act_buf,
                                 int64_t L, int64_t O, int64_t I, int8_t* gy_codes,
                                 float* gy_scale, int32_t* acc, void* stream) {
  Config c;
  hot_status st = resolve_config(cfg, &c);
  if (st != HOT_OK) return st;
  if (!ws || (acc && !act_buf)) return HOT_ERR_ARG;
  if (!tok_shape_ok(c, L, O) || !tok_shape_ok(c, L, I)) return HOT_ERR_SHAPE;
  const GwLayout g = gw_layout(c, L, O, I);
  const ActLayout a = act_layout(c, L, I);
  hipStream_t s = (hipStream_t)stream;
  uint8_t* base = (uint8_t*)ws;
  if (gy_codes) HOT_TRY(launch_unpack(base + g.qg, O, g.Lr, g.pitch, c.gw_bits, 1, gy_codes, s));
  if (gy_scale) HOT_TRY(hipMemcpyAsync(gy_scale, base + g.scalars, 4, hipMemcpyDeviceToDevice, s));
  if (acc)
    HOT_TRY(gemm(c, base + g.qg, (const uint8_t*)act_buf + a.codes, O, I, g.pitch, c.gw_bits, base,
                 g.partial, acc, nullptr, nullptr, 0, nullptr, c.n, s));
  return HOT_OK;
}

hot_status hot_debug_fused_operands(const hot_config* cfg, void* ws, const void* act_buf,
                                    int64_t L, int64_t O, int64_t I, hot_quantizer gy_quantizer,
                                    int8_t* gy_codes, float* gy_scales, int8_t* w_codes,
                                    float* w_scale, int32_t* acc_gx, int8_t* gyT_codes,
                                    float* gyT_scale, int32_t* acc_gw, void* stream) {
  Config c;
  hot_status st = resolve_config(cfg, &c);
  if (st != HOT_OK) return st;
  if (!ws || (acc_gw && !act_buf)) return HOT_ERR_ARG;
  if (!gx_shape_ok(c, L, O, I) || !tok_shape_ok(c, L, O) || !tok_shape_ok(c, L, I)) return HOT_ERR_SHAPE;
  if (!shared_gy_passes(c, L, O)) return HOT_ERR_UNIMPLEMENTED;
  st = hot_debug_gx_operands(cfg, ws, L, O, I, gy_quantizer, gy_codes, gy_scales, w_codes, w_scale,
                             acc_gx, stream);
  if (st != HOT_OK) return st;
  const FusedLayout f = fused_layout(c, L, O, I);
  const ActLayout a = act_layout(c, L, I);
  hipStream_t s = (hipStream_t)stream;
  uint8_t* base = (uint8_t*)ws;
  if (gyT_codes) HOT_TRY(launch_unpack(base + f.qgh, O, f.gw.Lr, f.gw.pitch, 8, 1, gyT_codes, s));
  if (gyT_scale) HOT_TRY(hipMemcpyAsync(gyT_scale, base + f.s_gh, 4, hipMemcpyDeviceToDevice, s));
  if (acc_gw)
    HOT_TRY(gemm(c, base + f.qgh, (const uint8_t*)act_buf + a.codes, O, I, f.gw.pitch, 8, base, f.partial,
                 acc_gw, nullptr, nullptr, 0, nullptr, c.n, s));
  return HOT_OK;
}

}  // extern "C"
