// Row-direction block Walsh-Hadamard transform fused with abs-max and quantisation
// (device code; launchers in row_quant.hip): the g_y operand of the g_x path (Sec. 5.1)
// and the first half of quantizer selection (Sec. 5.2.2).
//
// Each row is read once with fully coalesced 16-byte loads and kept in
// registers.  A lane holds 4 consecutive elements, so butterfly stages h = 1, 2
// are in-lane and stages h = 4 .. n/2 exchange with lanes id^1, id^2, id^4, id^8
// (DPP / ds_swizzle).  HBM-bound: 4 bytes read and bits/8 bytes written per
// element.
#pragma once
#include "hot_device.h"

namespace hot {


__device__ __forceinline__ void store_codes4(uint8_t* row_codes, int e, const float4& q, float inv,
                                             int qmax, int bits, int rounding) {
  const int c0 = quant_code(q.x, inv, qmax, rounding), c1 = quant_code(q.y, inv, qmax, rounding);
  const int c2 = quant_code(q.z, inv, qmax, rounding), c3 = quant_code(q.w, inv, qmax, rounding);
  if (bits == 4) {
    const unsigned p = (c0 & 0xF) | ((c1 & 0xF) << 4) | ((c2 & 0xF) << 8) | ((c3 & 0xF) << 12);
    *reinterpret_cast<uint16_t*>(row_codes + (e >> 1)) = (uint16_t)p;
  } else {
    *reinterpret_cast<uint32_t*>(row_codes + e) = pack4_codes8(c0, c1, c2, c3);
  }
}

struct RowQuantArgs {
  const float* t;
  int64_t rows;
  int cols, bits, rounding, mode;
  uint8_t* codes;
  int64_t pitch;
  float* scales;
  float* partials;
  int npartials;
};

// TPR threads per row (64: one wave per row, 4 rows per workgroup; 256: one row per
// workgroup), ITER float4 per thread, so a row of up to 4*TPR*ITER elements lives
// in registers.  Body for workgroup `bid` of `nbid` (the whole grid, or the trailing part
// of a grid whose first workgroups do unrelated work).
template <int N, int ITER, int TPR>
__device__ __forceinline__ void row_quant_body(const RowQuantArgs& a, const int64_t bid, const int64_t nbid) {
  const float* __restrict__ t = a.t;
  const int64_t rows = a.rows;
  const int cols = a.cols, bits = a.bits, rounding = a.rounding, mode = a.mode;
  uint8_t* __restrict__ codes = a.codes;
  const int64_t pitch = a.pitch;
  float* __restrict__ scales = a.scales;
  float* __restrict__ partials = a.partials;
  const int npartials = a.npartials;
  constexpr int RPB = 256 / TPR;
  __shared__ float s_max[4];
  const int tid = threadIdx.x;
  const int rl = tid / TPR, tr = tid % TPR;
  const int qmax = (1 << (bits - 1)) - 1;
  const int64_t nrb = (rows + RPB - 1) / RPB;
  const int valid_bytes = cols * bits / 8;
  float running = 0.0f;  // modes 1, 3: abs-max over all rows this thread's group saw
  float amax_tensor = 0.0f;
  if (mode == 2) amax_tensor = block_max_of(partials, npartials);

  for (int64_t rb0 = bid; rb0 < nrb; rb0 += nbid) {
    // the second pass of the per-tensor form starts where the first one ended: those rows are
    // what the memory-side cache still holds
    const int64_t rb = mode == 2 ? nrb - 1 - rb0 : rb0;
    const int64_t row = rb * RPB + rl;
    const bool row_ok = row < rows;
    const float4* src = reinterpret_cast<const float4*>(t + row * (int64_t)cols);
    float4 v[ITER];
    float m = 0.0f;
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
      const int e = (it * TPR + tr) * 4;
      v[it] = (row_ok && e < cols) ? src[it * TPR + tr] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
      fwht_row4<N>(v[it], tr);
      m = fmaxf(m, absmax4(v[it]));
    }
    float amax;
    if (mode == 2) {
      amax = amax_tensor;
    } else {
      m = wave_max(m);
      if constexpr (TPR == 256) {
        if ((tid & 63) == 0) s_max[tid >> 6] = m;
        __syncthreads();
        m = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));
        __syncthreads();
      }
      amax = m;
    }
    if (mode == 1 || mode == 3) {
      running = fmaxf(running, amax);
      if (mode == 3 && tr == 0 && row_ok) scales[row] = amax;
      continue;
    }
    if (mode == 0 && tr == 0 && row_ok) scales[row] = quant_scale(amax, qmax);
    const float inv = quant_inv(amax, qmax);
    if (row_ok) {
      uint8_t* row_codes = codes + row * pitch;
#pragma unroll
      for (int it = 0; it < ITER; ++it) {
        const int e = (it * TPR + tr) * 4;
        if (e < cols) store_codes4(row_codes, e, v[it], inv, qmax, bits, rounding);
      }
      for (int off = valid_bytes + 4 * tr; off < pitch; off += 4 * TPR)
        *reinterpret_cast<uint32_t*>(row_codes + off) = 0u;
    }
  }
  if (mode == 1 || mode == 3) {
    // every lane of a row group holds that group's maximum; combine the groups
    __syncthreads();
    if ((tid & 63) == 0) s_max[tid >> 6] = running;
    __syncthreads();
    if (tid == 0) partials[bid] = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));
  } else if (mode == 2 && bid == 0 && tid == 0) {
    scales[0] = quant_scale(amax_tensor, qmax);
  }
}

template <int N, int ITER, int TPR>
__global__ __launch_bounds__(256) void row_quant_kernel(const RowQuantArgs a) {
  row_quant_body<N, ITER, TPR>(a, blockIdx.x, gridDim.x);
}

}  // namespace hot
