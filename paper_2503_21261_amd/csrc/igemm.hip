// Launchers of the integer GEMM (kernel in igemm_kernel.h), the split-K reduction and
// the code unpacker used by the parity views.
#include <atomic>

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

// Tile configurations.  Three workgroup tiles exist: 128x128 (64x64 per wave, three
// workgroups per compute unit, so one workgroup's stores overlap the others' main
// loops, but the INT4 widening costs 6 vector instructions per matrix instruction and
// the vector pipe becomes the limit), 192x256 and 256x256 (96x128 / 128x128 per wave,
// one workgroup per unit, half the widening and LDS traffic per matrix instruction, but
// nothing hides the output stores and a partial last round idles units).  The choice
// minimises a cost model fitted to measurements on MI355X: rounds over the 256 units
// x (tile operations / sustained rate of that tile + unhidden store time).  INT8
// operands (twice the bytes per operation) take 128-byte K stages.  A GEMM with a small
// output and a long K (the g_w path) is split along K only as far as needed to give
// every unit a workgroup: each extra slice costs an int32 image of the output in HBM.
GemmPlan plan_gemm(int64_t M, int64_t N, int64_t k_bytes, int bits, bool allow_split) {
  struct Cand { int bm, bn; double tops; bool hides_stores; };
  static const Cand cands4[] = {{128, 128, 1900., true}, {192, 256, 2700., false}, {256, 256, 3200., false}};
  static const Cand cands8[] = {{128, 128, 1000., true}, {256, 256, 2200., false}};
  const Cand* cands = bits == 4 ? cands4 : cands8;
  const int ncand = bits == 4 ? 3 : 2;
  const double K = (double)k_bytes * (bits == 4 ? 2 : 1);
  GemmPlan p;
  p.split = 1;
  p.partial_bytes = 0;
  double best = 1e30;
  for (int c = 0; c < ncand; ++c) {
    const int64_t tiles = ceil_div(M, cands[c].bm) * ceil_div(N, cands[c].bn);
    const double rounds = (double)ceil_div(tiles, 256);
    const double ops = 2.0 * cands[c].bm * cands[c].bn * K;
    double t = ops / (cands[c].tops * 1e12 / 256);
    if (!cands[c].hides_stores) t += 4.0 * cands[c].bm * cands[c].bn / (5.5e12 / 256);
    t *= rounds;
    if (t < best) {
      best = t;
      p.bm = cands[c].bm;
      p.bn = cands[c].bn;
      p.tiles = tiles;
    }
  }
  p.bkb = bits == 4 ? 64 : 128;
  if (allow_split && p.bm == 128) {
    int64_t s = 256 / p.tiles;
    const int64_t nk = k_bytes / p.bkb;
    if (s > nk / 4) s = nk / 4;   // at least 4 stages per slice
    if (s >= 2) {
      p.split = (int)ceil_div(nk, ceil_div(nk, s));   // no empty slice
      p.partial_bytes = (size_t)p.tiles * p.split * 128 * 128 * 4;
    }
  }
  return p;
}

namespace {

template <int BM, int BN, int BKB, bool INT4, bool BF16 = false>
hipError_t launch_tile(GemmArgs g, int64_t k_bytes, hipStream_t s, int gemm_stage, int reduce_stage) {
  if (BF16 && g.split != 1) return hipErrorInvalidValue;
  g.nk_total = (int)(k_bytes / BKB);
  g.stages_per_split = (int)ceil_div(g.nk_total, g.split);
  g.tiles_m = (int)ceil_div(g.M, BM);
  g.tiles_n = (int)ceil_div(g.N, BN);
  const size_t lds = 2 * (size_t)(BM + BN) * BKB;
  auto kern = igemm_kernel<BM, BN, 2, 2, BKB, INT4, BF16>;
  static std::atomic<bool> attr_set{false};  // per instantiation; setting it twice is harmless
  if (!attr_set.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set.store(true, std::memory_order_release);
  }
  const dim3 grid((unsigned)((int64_t)g.tiles_m * g.tiles_n), 1, (unsigned)g.split);
  if (gemm_stage >= 0) stage_begin(gemm_stage, s);
  kern<<<grid, dim3(256), lds, s>>>(g);
  if (gemm_stage >= 0) stage_end(gemm_stage, s);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || g.split == 1) return e;
  const unsigned blocks = (unsigned)((int64_t)g.tiles_m * g.tiles_n * (BM * BN / 256 / 16));
  if (reduce_stage >= 0) stage_begin(reduce_stage, s);
  splitk_image_reduce_kernel<BM, BN, 2, 2><<<dim3(blocks), dim3(256), 0, s>>>(g);
  if (reduce_stage >= 0) stage_end(reduce_stage, s);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_igemm(const uint8_t* A, const uint8_t* B, int64_t M, int64_t N, int64_t k_bytes,
                        int64_t pitch, int bits, const GemmPlan& plan, int32_t* partial,
                        int32_t* out_i32, float* out_f32, const float* row_scale,
                        int row_stride, const float* col_scale, int n, hipStream_t s,
                        int gemm_stage, int reduce_stage) {
  if (M <= 0 || N <= 0) return hipSuccess;
  if (plan.split > 1 && !partial) return hipErrorInvalidValue;
  GemmArgs g;
  g.A = A;
  g.B = B;
  g.M = (int)M;
  g.N = (int)N;
  g.pitch = pitch;
  g.out_i32 = out_i32;
  g.out_f32 = out_i32 ? nullptr : out_f32;  // int32 wins; callers ask one at a time
  g.split = plan.split;
  g.partial = partial;
  g.row_scale = row_scale;
  g.row_stride = row_stride;
  g.col_scale = col_scale;
  g.inv_n = 1.0f / (float)n;
  const int gs = gemm_stage, rs = reduce_stage;
  if (bits == 16) {
    if (plan.bm == 256) return launch_tile<256, 256, 128, false, true>(g, k_bytes, s, gs, rs);
    if (plan.bm == 128) return launch_tile<128, 128, 128, false, true>(g, k_bytes, s, gs, rs);
    return hipErrorInvalidValue;
  }
  if (plan.bm == 256)
    return bits == 4 ? launch_tile<256, 256, 64, true>(g, k_bytes, s, gs, rs)
                     : launch_tile<256, 256, 128, false>(g, k_bytes, s, gs, rs);
  if (plan.bm == 192 && bits == 4) return launch_tile<192, 256, 64, true>(g, k_bytes, s, gs, rs);
  if (plan.bm == 128)
    return bits == 4 ? launch_tile<128, 128, 64, true>(g, k_bytes, s, gs, rs)
                     : launch_tile<128, 128, 128, false>(g, k_bytes, s, gs, rs);
  return hipErrorInvalidValue;
}

}  // namespace hot
