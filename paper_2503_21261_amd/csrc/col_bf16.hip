// bfloat16 variant of the token-direction low-rank operands of the g_w path (Sec. 5.2 with
// the INT8 quantiser replaced by a rounding to bfloat16, the option Sec. 4.2 motivates: g_w
// is the gradient that suffers from quantisation).  Same block transform, row selection
// and transposed K-contiguous write as the column quantiser, but no scale: one pass.
#include "col_quant_kernel.h"

namespace hot {

// fp32 -> bfloat16 pattern, round to nearest even (finite inputs).
__device__ __forceinline__ uint32_t bf16_rne(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

template <int N, int KIND>
__global__ __launch_bounds__(256) void col_bf16_kernel(const float* __restrict__ x, RowTiling rt,
                                                       int64_t C, KeepMap map, int r, int kbw,
                                                       uint8_t* __restrict__ out, int64_t pitch,
                                                       float* __restrict__ scale) {
  static_assert(KIND == kKeepLowHalf || KIND == kKeepGeneric, "kept list");
  constexpr int CT = 64;
  extern __shared__ __align__(16) uint8_t tile[];
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int bpb = 2 * (KIND == kKeepLowHalf ? N / 2 : r);   // bytes per block and column
  const int TB = 4 * kbw * bpb, TBP = TB + 4;
  const int64_t nblk = rt.nblk;
  const int64_t tiles_x = (C + CT - 1) / CT;
  const int64_t tx = blockIdx.x % tiles_x, ty = blockIdx.x / tiles_x;
  const int64_t c0 = tx * CT + lane;
  const bool col_ok = c0 < C;
  if (blockIdx.x == 0 && tid == 0) *scale = 1.0f;   // the GEMM epilogue multiplies by it
  if ((ty + 1) * 4 * kbw > nblk) {   // slots of blocks past the end read back as +0
    for (int i = tid; i < CT * TBP / 4; i += 256) reinterpret_cast<uint32_t*>(tile)[i] = 0u;
    __syncthreads();
  }
  for (int kb = 0; kb < kbw; ++kb) {
    const int slot = w * kbw + kb;
    const int64_t gb = ty * 4 * kbw + slot;
    if (gb >= nblk || !col_ok) continue;
    float v[1][kept_vals<N, KIND>()];
    int64_t first;
    int valid;
    block_rows<N>(rt, gb, first, valid);
    load_block_kept<N, 1, KIND>(x + first * C + c0, C, valid, v);
    uint8_t* dst = tile + lane * TBP + slot * bpb;
    if constexpr (KIND == kKeepLowHalf) {
#pragma unroll
      for (int j2 = 0; j2 < N / 4; ++j2) {
        const uint32_t lo = bf16_rne(v[0][lowpass_row(N, 2 * j2) >> 1]);
        const uint32_t hi = bf16_rne(v[0][lowpass_row(N, 2 * j2 + 1) >> 1]);
        reinterpret_cast<uint32_t*>(dst)[j2] = lo | (hi << 16);
      }
    } else {
#pragma unroll
      for (int k = 0; k < N; ++k) {
        const int p = map.pos[k];
        if (p >= 0) reinterpret_cast<uint16_t*>(dst)[p] = (uint16_t)bf16_rne(v[0][k]);
      }
    }
  }
  __syncthreads();
  write_out_tile<1>(tile, TB, TBP, tx, ty, nblk, kbw, C, pitch, out);
}

namespace {
template <int N>
hipError_t launch_n(const float* x, const RowTiling& rt, int64_t C, const Config& cfg, uint8_t* out,
                    int64_t pitch, float* scale, hipStream_t s) {
  const bool low = cfg.lowpass_default && cfg.r * 2 == cfg.n;
  const int bpb = 2 * cfg.r;
  const int64_t nblk = rt.nblk;
  int kbw = 128 / bpb;
  kbw = kbw < 1 ? 1 : (kbw > 8 ? 8 : kbw);
  auto tiles = [&](int k) { return ceil_div(C, 64) * ceil_div(nblk, 4 * k); };
  while (tiles(kbw) < 512 && kbw > 1) kbw /= 2;
  const size_t lds = (size_t)64 * (4 * kbw * bpb + 4);
  const dim3 grid((unsigned)tiles(kbw));
  if (low) col_bf16_kernel<N, kKeepLowHalf><<<grid, dim3(256), lds, s>>>(x, rt, C, cfg.map, cfg.r, kbw, out, pitch, scale);
  else col_bf16_kernel<N, kKeepGeneric><<<grid, dim3(256), lds, s>>>(x, rt, C, cfg.map, cfg.r, kbw, out, pitch, scale);
  return hipGetLastError();
}
}  // namespace

hipError_t launch_col_bf16(const float* x, const RowTiling& rt, int64_t C, const Config& cfg, uint8_t* out,
                           int64_t pitch, float* scale, hipStream_t s, int stage) {
  if (rt.nblk <= 0 || C <= 0) return hipSuccess;
  hipError_t e = hipErrorInvalidValue;
  stage_begin(stage, s);
  switch (cfg.n) {
    case 16: e = launch_n<16>(x, rt, C, cfg, out, pitch, scale, s); break;
    case 32: e = launch_n<32>(x, rt, C, cfg, out, pitch, scale, s); break;
    case 64: e = launch_n<64>(x, rt, C, cfg, out, pitch, scale, s); break;
  }
  stage_end(stage, s);
  return e;
}

}  // namespace hot
