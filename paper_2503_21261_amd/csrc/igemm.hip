// Integer GEMM on the CDNA4 matrix cores with fused dequantisation:
//   C[M x N] = A[M x K] . B[N x K]^T,  both operands K-contiguous code rows.
// g_x path (Sec. 5.1): A = Q(g_y H^T) [L x O], B = Q(H w)^T [I x O], INT4.
// g_w path (Sec. 5.2): A = Q(HLA(g_y))^T [O x L'], B = x_hat^T [I x L'], INT8.
//
// v_mfma_i32_32x32x32_i8: a lane supplies 16 consecutive K bytes of row (lane%32)
// for A and of column (lane%32) for B, K group lane/32; the same K mapping is
// used for both operands, so only "same bytes on both sides" matters.  gfx950 has
// no INT4 matrix instruction: packed nibbles are widened in registers to
// 16 x code (low nibble: (d << 4) & 0xF0F0F0F0, high nibble: d & 0xF0F0F0F0, both
// sign-correct as int8), so the accumulator is exactly 256 x the true sum and is
// shifted back in the epilogue.  Packing halves global and LDS traffic.
//
// The dequantisation of Sec. 4.3 / Supp. F (a diagonal scaling) is the epilogue:
// out = acc * row_scale[m] * col_scale / n.
#include "hot_device.h"
#include "hot_host.h"

namespace hot {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));

constexpr int kBK = 64;        // K bytes per pipeline stage
constexpr int kLdsPitch = 80;  // 64 + 16: conflict-free 16-byte row reads

template <int BM, int BN, bool INT4>
__global__ __launch_bounds__(256) void igemm_kernel(
    const uint8_t* __restrict__ A, const uint8_t* __restrict__ B, int M, int N, int nk_total,
    int64_t pitch, int stages_per_split, int tiles_m, int32_t* __restrict__ out_i32,
    float* __restrict__ out_f32, const float* __restrict__ row_scale, int row_stride,
    const float* __restrict__ col_scale, float inv_n) {
  constexpr int WM = BM / 2, WN = BN / 2;  // 2 x 2 waves
  constexpr int TM = WM / 32, TN = WN / 32;
  __shared__ __align__(16) uint8_t As[2][BM * kLdsPitch];
  __shared__ __align__(16) uint8_t Bs[2][BN * kLdsPitch];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int tm = blockIdx.x % tiles_m, tn = blockIdx.x / tiles_m;
  const int m0 = tm * BM, n0 = tn * BN;
  const int wm0 = (wave & 1) * WM, wn0 = (wave >> 1) * WN;
  const int k_begin = blockIdx.z * stages_per_split;
  int k_end = k_begin + stages_per_split;
  if (k_end > nk_total) k_end = nk_total;

  // global -> register staging: 4 threads x 16 bytes cover one 64-byte K slice of a row
  const int lr = tid >> 2, lseg = (tid & 3) * 16;
  const uint8_t* a_src[BM / 64];
  const uint8_t* b_src[BN / 64];
#pragma unroll
  for (int p = 0; p < BM / 64; ++p) {
    int row = m0 + lr + 64 * p;
    row = row < M ? row : M - 1;  // rows past the edge re-read the last row; never stored
    a_src[p] = A + (int64_t)row * pitch + lseg;
  }
#pragma unroll
  for (int p = 0; p < BN / 64; ++p) {
    int row = n0 + lr + 64 * p;
    row = row < N ? row : N - 1;
    b_src[p] = B + (int64_t)row * pitch + lseg;
  }
  v4i ra[BM / 64], rb[BN / 64];
  auto load_stage = [&](int kt) {
    const int64_t off = (int64_t)kt * kBK;
#pragma unroll
    for (int p = 0; p < BM / 64; ++p) ra[p] = *reinterpret_cast<const v4i*>(a_src[p] + off);
#pragma unroll
    for (int p = 0; p < BN / 64; ++p) rb[p] = *reinterpret_cast<const v4i*>(b_src[p] + off);
  };
  auto store_stage = [&](int buf) {
#pragma unroll
    for (int p = 0; p < BM / 64; ++p)
      *reinterpret_cast<v4i*>(&As[buf][(lr + 64 * p) * kLdsPitch + lseg]) = ra[p];
#pragma unroll
    for (int p = 0; p < BN / 64; ++p)
      *reinterpret_cast<v4i*>(&Bs[buf][(lr + 64 * p) * kLdsPitch + lseg]) = rb[p];
  };

  v16i acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

  const int frag_row = lane & 31, frag_k = (lane >> 5) * 16;

  if (k_begin < k_end) {
    load_stage(k_begin);
    store_stage(0);
    __syncthreads();
    for (int kt = k_begin; kt < k_end; ++kt) {
      const int buf = (kt - k_begin) & 1;
      if (kt + 1 < k_end) load_stage(kt + 1);
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        v4i a[TM], b[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
          a[i] = *reinterpret_cast<const v4i*>(
              &As[buf][(wm0 + i * 32 + frag_row) * kLdsPitch + ks * 32 + frag_k]);
#pragma unroll
        for (int j = 0; j < TN; ++j)
          b[j] = *reinterpret_cast<const v4i*>(
              &Bs[buf][(wn0 + j * 32 + frag_row) * kLdsPitch + ks * 32 + frag_k]);
        if constexpr (INT4) {
          v4i alo[TM], ahi[TM], blo[TN], bhi[TN];
#pragma unroll
          for (int i = 0; i < TM; ++i) {
            alo[i] = (v4i)(((v4u)a[i] << 4) & 0xF0F0F0F0u);
            ahi[i] = (v4i)((v4u)a[i] & 0xF0F0F0F0u);
          }
#pragma unroll
          for (int j = 0; j < TN; ++j) {
            blo[j] = (v4i)(((v4u)b[j] << 4) & 0xF0F0F0F0u);
            bhi[j] = (v4i)((v4u)b[j] & 0xF0F0F0F0u);
          }
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
              acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(alo[i], blo[j], acc[i][j], 0, 0, 0);
              acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ahi[i], bhi[j], acc[i][j], 0, 0, 0);
            }
        } else {
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
              acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i][j], 0, 0, 0);
        }
      }
      if (kt + 1 < k_end) store_stage(buf ^ 1);
      __syncthreads();
    }
  }

  // Epilogue.  Accumulator register v of a 32x32 tile: row 8*(v/4) + 4*(lane/32) + v%4,
  // column lane%32, so each register is stored as 32-float (128-byte) row segments.
  const float cs = out_f32 ? (*col_scale) * inv_n : 0.0f;
  const int64_t zoff = out_i32 ? (int64_t)blockIdx.z * M * (int64_t)N : 0;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int m = m0 + wm0 + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
      if (m >= M) continue;
      const float rs = out_f32 ? row_scale[(int64_t)m * row_stride] * cs : 0.0f;
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int n = n0 + wn0 + j * 32 + (lane & 31);
        if (n >= N) continue;
        int c = acc[i][j][v];
        if constexpr (INT4) c >>= 8;
        const int64_t o = (int64_t)m * N + n;
        if (out_f32) out_f32[o] = (float)c * rs;
        else out_i32[zoff + o] = c;
      }
    }
  }
}

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

int gemm_split_k(int64_t M, int64_t N, int64_t k_bytes) {
  const int64_t tiles = ceil_div(M, 128) * ceil_div(N, 128);
  const int64_t nk = k_bytes / kBK;
  int64_t s = ceil_div(1024, tiles);        // aim for >= 4 workgroups per compute unit
  if (s > nk / 8) s = nk / 8;               // keep at least 8 stages per slice
  if (s > 64) s = 64;
  return s < 1 ? 1 : (int)s;
}

hipError_t launch_igemm(const uint8_t* A, const uint8_t* B, int64_t M, int64_t N, int64_t k_bytes,
                        int64_t pitch, int bits, int split_k, int32_t* partial, int32_t* out_i32,
                        float* out_f32, const float* row_scale, int row_stride,
                        const float* col_scale, int n, hipStream_t s, int gemm_stage,
                        int reduce_stage) {
  if (M <= 0 || N <= 0) return hipSuccess;
  constexpr int BM = 128, BN = 128;
  const int nk = (int)(k_bytes / kBK);
  const int tiles_m = (int)ceil_div(M, BM), tiles_n = (int)ceil_div(N, BN);
  if (split_k < 1 || partial == nullptr) split_k = 1;
  const int sps = (int)ceil_div(nk, split_k);
  const float inv_n = 1.0f / (float)n;
  const dim3 grid((unsigned)((int64_t)tiles_m * tiles_n), 1, (unsigned)split_k);
  int32_t* k_i32 = split_k > 1 ? partial : out_i32;
  float* k_f32 = split_k > 1 ? nullptr : out_f32;
  if (split_k == 1 && out_i32 && out_f32) k_f32 = nullptr;  // int32 wins; caller asks one at a time
  if (gemm_stage >= 0) stage_begin(gemm_stage, s);
  if (bits == 4)
    igemm_kernel<BM, BN, true><<<grid, dim3(256), 0, s>>>(A, B, (int)M, (int)N, nk, pitch, sps, tiles_m,
                                                         k_i32, k_f32, row_scale, row_stride,
                                                         col_scale, inv_n);
  else
    igemm_kernel<BM, BN, false><<<grid, dim3(256), 0, s>>>(A, B, (int)M, (int)N, nk, pitch, sps, tiles_m,
                                                          k_i32, k_f32, row_scale, row_stride,
                                                          col_scale, inv_n);
  if (gemm_stage >= 0) stage_end(gemm_stage, s);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || split_k == 1) return e;
  int64_t blocks = ceil_div(M * N, 256);
  if (blocks > 4096) blocks = 4096;
  if (reduce_stage >= 0) stage_begin(reduce_stage, s);
  splitk_reduce_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(
      partial, split_k, M, N, out_i32, out_i32 ? nullptr : out_f32, row_scale, row_stride,
      col_scale, inv_n);
  if (reduce_stage >= 0) stage_end(reduce_stage, s);
  return hipGetLastError();
}

}  // namespace hot
