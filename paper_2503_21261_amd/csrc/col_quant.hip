// Column-direction block Walsh-Hadamard transform with row selection (HLA,
// Sec. 3.3 Eq. 5), tensor-wide abs-max quantisation and a transposed,
// K-contiguous write.  Serves three operands:
//   - w rotated along O for the g_x path (Sec. 5.1): full rank, INT4/INT8;
//   - x compressed along L at forward time (Sec. 5.2.1): r of n rows, INT8;
//   - g_y compressed along L for the g_w path (Sec. 5.2): r of n rows, INT8.
//
// A lane owns VEC adjacent columns and holds the n rows of one block in
// registers (n coalesced row loads in flight), so every butterfly is in-register.
// Four waves take different blocks; their codes are gathered in LDS as
// [column][reduced-row bytes] and written out as contiguous runs per column, so
// the matrix-core GEMM that follows reads both operands K-contiguous and nothing
// is ever transposed in a separate pass.  HBM-bound: the tensor-wide scale forces
// two reads of the input (abs-max pass, quantise pass).
#include "hot_device.h"
#include "hot_host.h"

namespace hot {

template <int VEC> struct VecT;
template <> struct VecT<1> { using type = float; };
template <> struct VecT<2> { using type = float2; };
template <> struct VecT<4> { using type = float4; };

template <int VEC>
__device__ __forceinline__ void unpack_vec(const typename VecT<VEC>::type& q, float (&o)[VEC]) {
  if constexpr (VEC == 1) { o[0] = q; }
  else if constexpr (VEC == 2) { o[0] = q.x; o[1] = q.y; }
  else { o[0] = q.x; o[1] = q.y; o[2] = q.z; o[3] = q.w; }
}

// mode 1: abs-max of kept values -> atomic max.  mode 2: quantise + transposed write.
// grid.x = column tiles of CT = 64*VEC, grid.y = row tiles of 4*kbw blocks.
template <int N, int VEC>
__global__ __launch_bounds__(256) void col_quant_kernel(
    const float* __restrict__ x, int64_t R, int64_t C, KeepMap map, int r, int bits, int rounding,
    int mode, int kbw, uint8_t* __restrict__ codes, int64_t pitch, float* __restrict__ scale,
    unsigned* __restrict__ amax_bits) {
  using VT = typename VecT<VEC>::type;
  constexpr int CT = 64 * VEC;
  extern __shared__ __align__(16) uint8_t tile[];  // mode 2: [CT][TBP]
  __shared__ float s_max[4];

  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int qmax = (1 << (bits - 1)) - 1;
  const int bpb = bits == 4 ? N / 2 : r;   // code bytes one block contributes per column
  const int TB = 4 * kbw * bpb;            // code bytes per column in this tile
  const int TBP = TB + 4;
  const int64_t nblk = R / N;
  const int64_t c0 = (int64_t)blockIdx.x * CT + lane * VEC;
  const bool col_ok = c0 < C;

  float inv = 0.0f;
  if (mode == 2) {
    const float amax = __uint_as_float(*amax_bits);
    inv = quant_inv(amax, qmax);
    if (blockIdx.x == 0 && blockIdx.y == 0 && tid == 0) *scale = quant_scale(amax, qmax);
    for (int i = tid; i < CT * TBP / 4; i += 256) reinterpret_cast<uint32_t*>(tile)[i] = 0u;
    __syncthreads();
  }

  float m = 0.0f;
  for (int kb = 0; kb < kbw; ++kb) {
    const int slot = w * kbw + kb;
    const int64_t gb = (int64_t)blockIdx.y * 4 * kbw + slot;
    if (gb >= nblk || !col_ok) continue;
    float v[VEC][N];
    {
      const float* src = x + gb * N * C + c0;
      VT q[N];
#pragma unroll
      for (int k = 0; k < N; ++k) q[k] = *reinterpret_cast<const VT*>(src + (int64_t)k * C);
#pragma unroll
      for (int k = 0; k < N; ++k) {
        float o[VEC];
        unpack_vec<VEC>(q[k], o);
#pragma unroll
        for (int vi = 0; vi < VEC; ++vi) v[vi][k] = o[vi];
      }
    }
#pragma unroll
    for (int vi = 0; vi < VEC; ++vi) fwht_regs<N>(v[vi]);

    if (mode == 1) {
#pragma unroll
      for (int k = 0; k < N; ++k)
        if (map.pos[k] >= 0) {
#pragma unroll
          for (int vi = 0; vi < VEC; ++vi) m = fmaxf(m, fabsf(v[vi][k]));
        }
    } else {
      uint8_t* dst = tile + (lane * VEC) * TBP + slot * bpb;
      if (bits == 4) {
#pragma unroll
        for (int k = 0; k < N; k += 2) {
#pragma unroll
          for (int vi = 0; vi < VEC; ++vi) {
            const int lo = quant_code(v[vi][k], inv, qmax, rounding);
            const int hi = quant_code(v[vi][k + 1], inv, qmax, rounding);
            dst[vi * TBP + (k >> 1)] = (uint8_t)((lo & 0xF) | ((hi & 0xF) << 4));
          }
        }
      } else {
#pragma unroll
        for (int k = 0; k < N; ++k) {
          const int p = map.pos[k];
          if (p >= 0) {
#pragma unroll
            for (int vi = 0; vi < VEC; ++vi)
              dst[vi * TBP + p] = (uint8_t)quant_code(v[vi][k], inv, qmax, rounding);
          }
        }
      }
    }
  }

  if (mode == 1) {
    m = wave_max(m);
    if (lane == 0) s_max[w] = m;
    __syncthreads();
    if (tid == 0)
      atomic_absmax(amax_bits, fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3])));
    return;
  }

  __syncthreads();
  // Contiguous runs per column; the last row tile also zero-fills up to the pitch.
  const int64_t tile_off = (int64_t)blockIdx.y * TB;
  int64_t cover = (blockIdx.y == gridDim.y - 1) ? pitch - tile_off : TB;
  if (cover > pitch - tile_off) cover = pitch - tile_off;
  const int cdw = (int)(cover >> 2), tdw = TB >> 2;
  for (int idx = tid; idx < CT * cdw; idx += 256) {
    const int col = idx / cdw, dw = idx - col * cdw;
    const int64_t c = (int64_t)blockIdx.x * CT + col;
    if (c < C) {
      const uint32_t val = dw < tdw ? *reinterpret_cast<const uint32_t*>(tile + col * TBP + 4 * dw) : 0u;
      *reinterpret_cast<uint32_t*>(codes + c * pitch + tile_off + 4 * dw) = val;
    }
  }
}

namespace {

template <int N, int VEC>
hipError_t launch_cq(const float* x, int64_t R, int64_t C, const KeepMap& map, int r, int bits,
                     int rounding, int mode, uint8_t* codes, int64_t pitch, float* scale,
                     unsigned* amax_bits, hipStream_t s) {
  const int bpb = bits == 4 ? N / 2 : r;
  int kbw = 32 / bpb;
  kbw = kbw < 1 ? 1 : (kbw > 8 ? 8 : kbw);
  const int TB = 4 * kbw * bpb;
  const int64_t nblk = R / N;
  const dim3 grid((unsigned)ceil_div(C, 64 * VEC), (unsigned)ceil_div(nblk, 4 * kbw));
  const size_t lds = mode == 2 ? (size_t)(64 * VEC) * (TB + 4) : 0;
  col_quant_kernel<N, VEC><<<grid, dim3(256), lds, s>>>(x, R, C, map, r, bits, rounding, mode, kbw,
                                                       codes, pitch, scale, amax_bits);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_col_quant(const float* x, int64_t R, int64_t C, const Config& cfg, int r,
                            const KeepMap& map, int bits, int mode, uint8_t* codes,
                            int64_t pitch, float* scale, unsigned* amax_bits, hipStream_t s) {
  if (R <= 0 || C <= 0) return hipSuccess;
  const int rounding = cfg.rounding;
  // widest vector the column count allows, capped so 128 values stay in registers
  const int vmax = cfg.n == 64 ? 2 : 4;
  int vec = (C % 4 == 0) ? 4 : (C % 2 == 0 ? 2 : 1);
  if (vec > vmax) vec = vmax;
#define HOT_CQ(NN, VV) \
  return launch_cq<NN, VV>(x, R, C, map, r, bits, rounding, mode, codes, pitch, scale, amax_bits, s)
  switch (cfg.n * 8 + vec) {
    case 16 * 8 + 4: HOT_CQ(16, 4);
    case 16 * 8 + 2: HOT_CQ(16, 2);
    case 16 * 8 + 1: HOT_CQ(16, 1);
    case 32 * 8 + 4: HOT_CQ(32, 4);
    case 32 * 8 + 2: HOT_CQ(32, 2);
    case 32 * 8 + 1: HOT_CQ(32, 1);
    case 64 * 8 + 2: HOT_CQ(64, 2);
    case 64 * 8 + 1: HOT_CQ(64, 1);
  }
#undef HOT_CQ
  return hipErrorInvalidValue;
}

}  // namespace hot
