// Launch plan and launchers of the integer GEMM (kernel in igemm_kernel.h) and the code
// unpacker used by the parity views.
#include <atomic>
#include <chrono>

#include "hot_host.h"
#include "igemm_kernel.h"

namespace hot {

__global__ void unpack_kernel(const uint8_t* __restrict__ codes, int64_t rows, int64_t K,
                              int64_t pitch, int bits, int transpose, int8_t* __restrict__ out) {
  const int64_t total = rows * K;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t row = i / K, k = i - row * K;
    if (bits == 16) {   // two-byte elements (bfloat16 patterns) in, two-byte elements out
      reinterpret_cast<uint16_t*>(out)[transpose ? k * rows + row : i] =
          *reinterpret_cast<const uint16_t*>(codes + row * pitch + 2 * k);
      continue;
    }
    int c;
    if (bits == 4) {
      const int byte = codes[row * pitch + (k >> 1)];
      const int nib = (k & 1) ? (byte >> 4) : (byte & 0xF);
      c = (nib ^ 8) - 8;  // sign-extend 4 bits
    } else {
      c = (int8_t)codes[row * pitch + k];
    }
    out[transpose ? k * rows + row : i] = (int8_t)c;
  }
}

hipError_t launch_unpack(const uint8_t* codes, int64_t rows, int64_t K, int64_t pitch, int bits,
                         int transpose, int8_t* out, hipStream_t s) {
  if (rows <= 0 || K <= 0) return hipSuccess;
  int64_t blocks = ceil_div(rows * K, 256);
  if (blocks > 65536) blocks = 65536;
  unpack_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(codes, rows, K, pitch, bits, transpose, out);
  return hipGetLastError();
}

// Tile configurations.  Four workgroup tiles exist for INT4 operands: 128x128 (64x64 per
// wave, three workgroups per compute unit: prologue, matrix loop and epilogue of different
// workgroups overlap, but the INT4 widening costs 6 vector instructions per matrix
// instruction), 128x256 (64x128 per wave, two workgroups per unit), 192x256 and 256x256 (96x128
// / 128x128 per wave, one workgroup per unit: half the widening and LDS traffic per matrix
// instruction, but prologue (3 us) and epilogue (3 us of instructions, or the tile's bytes at
// the unit's share of the memory bandwidth when every unit stores at once) are exposed, and a
// partial last round idles units).  INT8 and bfloat16 operands (twice and four times the
// bytes per operation) take 128x128, whose LDS traffic (1 KB per matrix instruction) is its
// limit, or 256x256 with eight waves (64x128 per wave), and 128-byte K stages.  The choice
// minimises the cost model in plan_gemm.  A GEMM with a small output and a long K (the g_w
// path of ViT-sized layers) leaves most units idle with one workgroup per tile: its K range
// is split over several workgroups per tile, which hand their partial sums to the last one
// through the workspace.
namespace {
std::atomic<int> g_gemm_mode{0};   // 0: cost model, 1: never split K, s >= 2: s slices where possible
std::atomic<int> g_gemm_wait_us{200};

// Compute units the launch plans are made for: those of the MI355X.  A constant rather than
// a device query, so that workspace sizes are a function of the configuration and the shape
// alone; on a part with fewer units the plans stay correct (every wait for another workgroup is
// bounded), only less well fitted.
constexpr int kPlanComputeUnits = 256;
int compute_units() { return kPlanComputeUnits; }

// Most slices a 128x128-tile GEMM may be cut into: at least 4 K stages per slice, and no more
// image slots than the workspace has flags for.
int64_t max_split(int64_t tiles, int64_t nk) {
  int64_t s = nk / 4;
  if (s > 8) s = 8;
  while (s > 1 && tiles * (s - 1) > kMaxSplitSlots) --s;
  return s < 1 ? 1 : s;
}
// K split of the 256x256 INT8 tile (eight waves, one workgroup per compute unit) for an output
// of at most one such tile per unit: as many slices as there are units per tile, and only when
// a slice keeps at least 16 KB of K, so that the 256 KB accumulator images the owner collects
// are a small part of the work.  Measured: ViT-L fc1 g_w (64 tiles, K = 100864, 4 slices) 396 us
// against 483 us with 128x128 tiles in 2 slices; with 3152-byte slices (ViT-B qkv) 88 against
// 79 us, so short K stays on the small tile.  0: does not apply.
int64_t large_tile_split(int64_t M, int64_t N, int64_t k_bytes, int bits, int cus) {
  if (bits != 8) return 0;
  const int64_t tiles = ceil_div(M, 256) * ceil_div(N, 256);
  if (tiles > cus) return 0;
  int64_t s = cus / tiles;
  if (s > 8) s = 8;
  while (s > 1 && (k_bytes / s < 16384 || tiles * (s - 1) > kMaxSplitSlots)) --s;
  return s >= 2 ? s : 0;
}
}  // namespace

void set_gemm_mode(int mode) { g_gemm_mode.store(mode); }
void set_gemm_wait_us(int us) { g_gemm_wait_us.store(us); }

GemmPlan plan_gemm(int64_t M, int64_t N, int64_t k_bytes, int bits, bool scratch) {
  // Cost of a tile shape, fitted to measurements on MI355X (ten layer shapes from 512 to 201728
  // tokens, every INT4 tile timed on each; within 4 % of the measured time, and the measured
  // best tile or one within 2 % of it on all ten): a compute unit works through its share of
  // the tiles, each costing its operations at the rate the tile sustains plus its output bytes
  // at the rate its stores drain, plus a constant per launch.  The share is a whole number of
  // tiles while the resident workgroups (wgs per unit) take them in a few rounds, the last of
  // which idles units, and averages out over many rounds.
  struct Cand { int bm, bn, wgs; double us_per_mop, us_per_kb, us_launch; };
  static const Cand cands4[] = {{128, 128, 3, 0.0979, 0.0324, 4.3}, {128, 256, 2, 0.0880, 0.0310, 3.6},
                                {192, 256, 1, 0.0860, 0.0392, 5.6}, {256, 256, 1, 0.0821, 0.0385, 0.0}};
  static const Cand cands8[] = {{128, 128, 2, 0.2560, 0.0, 0.0}, {256, 256, 1, 0.1004, 0.0476, 0.0}};
  const Cand* cands = bits == 4 ? cands4 : cands8;
  const int ncand = bits == 4 ? 4 : 2;
  const double K = (double)k_bytes * (bits == 4 ? 2 : 1);
  const int cus = compute_units();
  GemmPlan p;
  p.split = 1;
  p.partial_bytes = 0;
  double best = 1e30;
  for (int c = 0; c < ncand; ++c) {
    const int64_t tiles = ceil_div(M, cands[c].bm) * ceil_div(N, cands[c].bn);
    const bool few_rounds = tiles <= 4 * (int64_t)cus * cands[c].wgs;
    const double per_cu = few_rounds ? (double)ceil_div(tiles, cus) : (double)tiles / cus;
    const double mops = 2.0 * cands[c].bm * cands[c].bn * K * 1e-6;
    const double kb = 4.0 * cands[c].bm * cands[c].bn / 1024.0;
    const double t = per_cu * (mops * cands[c].us_per_mop + kb * cands[c].us_per_kb) + cands[c].us_launch;
    if (t < best) {
      best = t;
      p.bm = cands[c].bm;
      p.bn = cands[c].bn;
      p.tiles = tiles;
    }
  }
  p.bkb = bits == 4 ? 64 : 128;
  const int mode = g_gemm_mode.load();
  if (mode >= 10) {   // a tile forced for measurement: 10 = 128x128, 11 = 192x256 (INT4 only), 12 = 256x256
    const int bm = mode == 10 ? 128 : (mode == 11 && bits == 4 ? 192 : 256);
    p.bm = bm;
    p.bn = bm == 128 ? 128 : 256;
    if (mode == 13 && bits == 4) { p.bm = 128; p.bn = 256; }
    p.tiles = ceil_div(M, p.bm) * ceil_div(N, p.bn);
    return p;
  }
  if (scratch && mode == 0) {
    const int64_t s = large_tile_split(M, N, k_bytes, bits, cus);
    if (s) {
      p.bm = p.bn = 256;
      p.tiles = ceil_div(M, 256) * ceil_div(N, 256);
      p.split = (int)s;
      p.partial_bytes = (size_t)p.tiles * (s - 1) * 256 * 256 * 4;
      return p;
    }
  }
  if (scratch && bits != 16 && p.bm == 128 && p.bn == 128 && mode != 1) {
    const int64_t nk = k_bytes / p.bkb, most = max_split(p.tiles, nk);
    // measured on MI355X (128x128 INT8 tiles, K of 50-200 stages): fastest with as many slices
    // as keep all workgroups resident at once, two per compute unit; a partial second round
    // costs more than the shorter slices gain
    int64_t s = mode >= 2 ? mode : (p.tiles <= cus ? 2 * cus / p.tiles : 1);
    if (s > most) s = most;
    if (s >= 2) {
      p.split = (int)s;
      p.partial_bytes = (size_t)p.tiles * (s - 1) * 128 * 128 * 4;
    }
  }
  return p;
}

size_t gemm_scratch_bytes(int64_t M, int64_t N, int64_t k_bytes, int bits) {
  if (bits == 16 || M <= 0 || N <= 0) return 0;
  const int64_t tiles = ceil_div(M, 128) * ceil_div(N, 128);
  const int64_t s = max_split(tiles, k_bytes / (bits == 4 ? 64 : 128));
  const size_t small = (size_t)tiles * (s - 1) * 128 * 128 * 4;
  const int64_t sl = large_tile_split(M, N, k_bytes, bits, compute_units());
  const size_t large = sl ? (size_t)(ceil_div(M, 256) * ceil_div(N, 256)) * (sl - 1) * 256 * 256 * 4 : 0;
  return small > large ? small : large;
}

namespace {


// Waves per workgroup: 2x2, except 4x2 for the 256x256 INT8 and bfloat16 tiles.  Four waves,
// alone on their SIMDs, cannot hide the LDS traffic of those operands (two and four times the
// bytes per matrix instruction of packed INT4); eight waves of 64x128 each, two per SIMD, keep
// the whole accumulator tile in the 512 registers per lane all the same.  Measured on the
// LLM-sized g_w GEMM: INT8 320 us against 364 us (4x4 waves: 351 us), bfloat16 640 against
// 688 us; the INT4 tile and the 128x128 tiles do not gain from more waves.
template <int BM, bool INT4, bool BF16>
constexpr int gemm_waves_m() { return (BM == 256 && !INT4) ? 4 : 2; }

template <int BM, int BN, int BKB, bool INT4, bool BF16, bool SPLITK>
hipError_t launch_kernel(const GemmArgs& g, unsigned grid, hipStream_t s, int gemm_stage) {
  const size_t lds = 2 * (size_t)(BM + BN) * BKB;
  constexpr int WM = gemm_waves_m<BM, INT4, BF16>();
  auto kern = igemm_kernel<BM, BN, WM, 2, BKB, INT4, BF16, SPLITK>;
  static std::atomic<bool> attr_set{false};  // per instantiation; setting it twice is harmless
  if (!attr_set.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set.store(true, std::memory_order_release);
  }
  if (gemm_stage >= 0) stage_begin(gemm_stage, s);
  kern<<<dim3(grid), dim3(64 * WM * 2), lds, s>>>(g);
  if (gemm_stage >= 0) stage_end(gemm_stage, s);
  return hipGetLastError();
}

template <int BM, int BN, int BKB, bool INT4, bool BF16 = false>
hipError_t launch_tile(GemmArgs g, int64_t k_bytes, int split, hipStream_t s, int gemm_stage) {
  g.nk_total = (int)(k_bytes / BKB);
  g.tiles_m = (int)ceil_div(g.M, BM);
  g.tiles_n = (int)ceil_div(g.N, BN);
  g.split = split;
  const int64_t tiles = (int64_t)g.tiles_m * g.tiles_n;
  if (split <= 1) return launch_kernel<BM, BN, BKB, INT4, BF16, false>(g, (unsigned)tiles, s, gemm_stage);
  if constexpr (BF16 || BM == 192 || BM != BN || (INT4 && BM != 128)) {
    return hipErrorInvalidValue;   // splits exist for the 128x128 tiles and the 256x256 INT8 tile
  } else {
    if (!g.partial || !g.flags || tiles * (split - 1) > kMaxSplitSlots) return hipErrorInvalidValue;
    g.tag = next_exchange_tag();   // the process-wide launch tag sequence
    // one rectangle of the tile grid per XCD where the grid divides evenly: the split that
    // fetches the fewest operand bytes (A row bands once per XCD column, B bands once per XCD row)
    g.xcd_cols = 0;
    if (BM == 128 && 8 % split == 0 && g.tiles_m % (8 / split) == 0) {
      // a slice per group of XCDs: the fewest operand bytes of all (ViT-B proj g_w, 36 tiles in
      // 8 slices: 50.5 -> 45 us; the 256x256 split measured slower this way, 385 against 360 us
      // on the ViT-L g_w GEMM, and keeps the rectangles)
      g.xcd_cols = -1;
    } else if (tiles % 8 == 0) {
      double best = 0.0;
      for (int rx = 1; rx <= 8; rx *= 2) {
        const int ry = 8 / rx;
        if (g.tiles_m % ry != 0 || g.tiles_n % rx != 0) continue;
        const double fetch = (double)g.M * rx + (double)g.N * ry;
        if (g.xcd_cols == 0 || fetch < best) {
          best = fetch;
          g.xcd_cols = rx;
        }
      }
    }
    // an image normally arrives before its owner has finished its own slice; the bound only
    // has to cover workgroups that start late: never less than the whole GEMM takes at 200 TOP/s
    int64_t wait_us = g_gemm_wait_us.load();
    const int64_t gemm_us = (int64_t)(2.0 * g.M * g.N * (double)k_bytes * (INT4 ? 2 : 1) / 200e6);
    if (wait_us > 0 && wait_us < gemm_us) wait_us = gemm_us;
    g.wait_ticks = wait_us < 0 ? 0 : wait_us * 100;
    return launch_kernel<BM, BN, BKB, INT4, false, true>(g, (unsigned)(tiles * split), s, gemm_stage);
  }
}

}  // namespace

hipError_t launch_igemm(const uint8_t* A, const uint8_t* B, int64_t M, int64_t N, int64_t k_bytes,
                        int64_t pitch, int bits, const GemmPlan& plan, int32_t* partial,
                        unsigned long long* flags, int32_t* out_i32, float* out_f32,
                        const float* row_scale, int row_stride, const float* col_scale, int n,
                        hipStream_t s, int gemm_stage, const unsigned long long* epoch) {
  if (M <= 0 || N <= 0) return hipSuccess;
  GemmArgs g;
  g.A = A;
  g.B = B;
  g.M = (int)M;
  g.N = (int)N;
  g.pitch = pitch;
  g.out_i32 = out_i32;
  g.out_f32 = out_i32 ? nullptr : out_f32;  // int32 wins; callers ask one at a time
  g.partial = partial;
  g.flags = flags;
  g.tag = 0;
  g.epoch = epoch;
  g.wait_ticks = 0;
  g.row_scale = row_scale;
  g.row_stride = row_stride;
  g.col_scale = col_scale;
  g.inv_n = 1.0f / (float)n;
  g.xcd_cols = 0;
  // measured on MI355X: streaming stores win for INT8 / bfloat16 operands and for INT4 GEMMs of
  // up to 3072 codes of K (ViT-B fc2 at 50432 tokens 167 -> 134 us, ViT-B fc1 at 12608 tokens
  // 44.5 -> 39.6 us), and lose 3 % at 4096 codes and a wide output (LLM down-projection)
  g.stream_out = (bits != 4 || k_bytes * 2 <= 3072) ? 1 : 0;
  const int gs = gemm_stage, sw = plan.split;
  if (bits == 16) {
    if (plan.bm == 256) return launch_tile<256, 256, 128, false, true>(g, k_bytes, sw, s, gs);
    if (plan.bm == 128) return launch_tile<128, 128, 128, false, true>(g, k_bytes, sw, s, gs);
    return hipErrorInvalidValue;
  }
  if (plan.bm == 256)
    return bits == 4 ? launch_tile<256, 256, 64, true>(g, k_bytes, sw, s, gs)
                     : launch_tile<256, 256, 128, false>(g, k_bytes, sw, s, gs);
  if (plan.bm == 192 && bits == 4) return launch_tile<192, 256, 64, true>(g, k_bytes, sw, s, gs);
  if (plan.bm == 128 && plan.bn == 256 && bits == 4) return launch_tile<128, 256, 64, true>(g, k_bytes, sw, s, gs);
  if (plan.bm == 128)
    return bits == 4 ? launch_tile<128, 128, 64, true>(g, k_bytes, sw, s, gs)
                     : launch_tile<128, 128, 128, false>(g, k_bytes, sw, s, gs);
  return hipErrorInvalidValue;
}

}  // namespace hot
