// Launchers of the integer GEMM (kernel in igemm_kernel.h), the split-K reduction and
// the code unpacker used by the parity views.
#include "hot_host.h"
#include "igemm_kernel.h"

namespace hot {

__global__ void unpack_kernel(const uint8_t* __restrict__ codes, int64_t rows, int64_t K,
                              int64_t pitch, int bits, int transpose, int8_t* __restrict__ out) {
  const int64_t total = rows * K;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t row = i / K, k = i - row * K;
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

// Tile configurations (measured on MI355X).  The 256x256 tile (one workgroup per compute
// unit, 128x128 per wave) has the best matrix-core duty cycle and the lowest operand
// traffic per operation, but needs >= 1024 tiles to balance 256 compute units.  Below
// that the 128x128 tile runs three workgroups per unit, which also overlaps one
// workgroup's output stores with the others' main loops; INT8 operands (twice the bytes
// per operation) take 128-byte K stages there.  A GEMM with a small output and a long K
// (the g_w path) is split along K only as far as needed to give every compute unit a
// workgroup: each extra slice costs a full int32 image of the output in HBM traffic.
GemmPlan plan_gemm(int64_t M, int64_t N, int64_t k_bytes, int bits, bool allow_split) {
  GemmPlan p;
  const int64_t t256 = ceil_div(M, 256) * ceil_div(N, 256);
  const int64_t t128 = ceil_div(M, 128) * ceil_div(N, 128);
  p.split = 1;
  p.partial_bytes = 0;
  if (t256 >= 1024) {
    p.bm = p.bn = 256;
    p.bkb = bits == 4 ? 64 : 128;
    p.tiles = t256;
    return p;
  }
  p.bm = p.bn = 128;
  p.bkb = bits == 4 ? 64 : 128;
  p.tiles = t128;
  if (allow_split) {
    int64_t s = 256 / t128;
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

template <int BM, int BN, int BKB, bool INT4>
hipError_t launch_tile(GemmArgs g, int64_t k_bytes, hipStream_t s, int gemm_stage, int reduce_stage) {
  g.nk_total = (int)(k_bytes / BKB);
  g.stages_per_split = (int)ceil_div(g.nk_total, g.split);
  g.tiles_m = (int)ceil_div(g.M, BM);
  g.tiles_n = (int)ceil_div(g.N, BN);
  const size_t lds = 2 * (size_t)(BM + BN) * (BKB + 16);
  auto kern = igemm_kernel<BM, BN, 2, 2, BKB, INT4>;
  static bool attr_set = false;  // per instantiation
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set = true;
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
  if (plan.bm == 256)
    return bits == 4 ? launch_tile<256, 256, 64, true>(g, k_bytes, s, gs, rs)
                     : launch_tile<256, 256, 128, false>(g, k_bytes, s, gs, rs);
  if (plan.bm == 128)
    return bits == 4 ? launch_tile<128, 128, 64, true>(g, k_bytes, s, gs, rs)
                     : launch_tile<128, 128, 128, false>(g, k_bytes, s, gs, rs);
  return hipErrorInvalidValue;
}

}  // namespace hot
