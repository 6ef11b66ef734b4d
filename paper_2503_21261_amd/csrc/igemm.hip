// Launchers of the integer GEMM (kernel in igemm_kernel.h), the split-K reduction and
// the code unpacker used by the parity views.
#include "hot_host.h"
#include "igemm_kernel.h"

namespace hot {

// Sums the K-slices of a split GEMM in slice order and applies the epilogue.
__global__ void splitk_reduce_kernel(const int32_t* __restrict__ partial, int split, int64_t M,
                                     int64_t N, int32_t* __restrict__ out_i32,
                                     float* __restrict__ out_f32,
                                     const float* __restrict__ row_scale, int row_stride,
                                     const float* __restrict__ col_scale, float inv_n) {
  const int64_t total = M * N;
  const float cs = out_f32 ? (*col_scale) * inv_n : 0.0f;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * blockDim.x) {
    int c = 0;
    for (int z = 0; z < split; ++z) c += partial[(int64_t)z * total + i];
    if (out_f32) out_f32[i] = (float)c * (row_scale[(i / N) * row_stride] * cs);
    else out_i32[i] = c;
  }
}

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

namespace {

// Tile configurations.  The 256x256 tile (one workgroup per compute unit, 128x128 per
// wave) has the best matrix-core duty cycle but needs many tiles to balance 256
// compute units; the 128x128 tile runs three workgroups per unit, which also overlaps
// one workgroup's output stores with the others' main loops.
struct TileCfg { int bm, bn, bkb; };

TileCfg pick_tile(int64_t M, int64_t N, int bits) {
  const int64_t big = ceil_div(M, 256) * ceil_div(N, 256);
  if (big >= 1024) return bits == 4 ? TileCfg{256, 256, 64} : TileCfg{256, 256, 128};
  return TileCfg{128, 128, 64};
}

template <int BM, int BN, int BKB, bool INT4>
hipError_t launch_tile(GemmArgs g, int64_t k_bytes, int split_k, hipStream_t s) {
  g.nk_total = (int)(k_bytes / BKB);
  g.stages_per_split = (int)ceil_div(g.nk_total, split_k);
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
  const dim3 grid((unsigned)((int64_t)g.tiles_m * g.tiles_n), 1, (unsigned)split_k);
  kern<<<grid, dim3(256), lds, s>>>(g);
  return hipGetLastError();
}

}  // namespace

int gemm_split_k(int64_t M, int64_t N, int64_t k_bytes) {
  const TileCfg t = pick_tile(M, N, 8);
  const int64_t tiles = ceil_div(M, t.bm) * ceil_div(N, t.bn);
  const int64_t nk = k_bytes / t.bkb;
  int64_t s = ceil_div(512, tiles);         // aim for >= 2 workgroups per compute unit
  if (s > nk / 8) s = nk / 8;               // keep at least 8 stages per slice
  if (s > 16) s = 16;
  return s < 1 ? 1 : (int)s;
}

hipError_t launch_igemm(const uint8_t* A, const uint8_t* B, int64_t M, int64_t N, int64_t k_bytes,
                        int64_t pitch, int bits, int split_k, int32_t* partial, int32_t* out_i32,
                        float* out_f32, const float* row_scale, int row_stride,
                        const float* col_scale, int n, hipStream_t s, int gemm_stage,
                        int reduce_stage) {
  if (M <= 0 || N <= 0) return hipSuccess;
  if (split_k < 1 || partial == nullptr) split_k = 1;
  GemmArgs g;
  g.A = A;
  g.B = B;
  g.M = (int)M;
  g.N = (int)N;
  g.pitch = pitch;
  g.out_i32 = split_k > 1 ? partial : out_i32;
  g.out_f32 = (split_k > 1 || out_i32) ? nullptr : out_f32;  // int32 wins; callers ask one at a time
  g.row_scale = row_scale;
  g.row_stride = row_stride;
  g.col_scale = col_scale;
  g.inv_n = 1.0f / (float)n;
  const TileCfg t = pick_tile(M, N, bits);
  if (gemm_stage >= 0) stage_begin(gemm_stage, s);
  hipError_t e;
  if (t.bm == 256) {
    e = bits == 4 ? launch_tile<256, 256, 64, true>(g, k_bytes, split_k, s)
                  : launch_tile<256, 256, 128, false>(g, k_bytes, split_k, s);
  } else {
    e = bits == 4 ? launch_tile<128, 128, 64, true>(g, k_bytes, split_k, s)
                  : launch_tile<128, 128, 64, false>(g, k_bytes, split_k, s);
  }
  if (gemm_stage >= 0) stage_end(gemm_stage, s);
  if (e != hipSuccess || split_k == 1) return e;
  int64_t blocks = ceil_div(M * N, 256);
  if (blocks > 4096) blocks = 4096;
  if (reduce_stage >= 0) stage_begin(reduce_stage, s);
  splitk_reduce_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(
      partial, split_k, M, N, out_i32, out_i32 ? nullptr : out_f32, row_scale, row_stride,
      col_scale, 1.0f / (float)n);
  if (reduce_stage >= 0) stage_end(reduce_stage, s);
  return hipGetLastError();
}

}  // namespace hot
