// Squared quantisation error of the rotated g_y under per-token and per-tensor
// scales: the measurement behind Layer-wise Quantizer Selection (Sec. 5.2.2).
// Calibration-time only; sums are double and combined in a fixed order so the
// result is reproducible run to run.
#include "hot_device.h"
#include "hot_host.h"

namespace hot {

__device__ __forceinline__ double sq_err(float t, float inv, float scale, int qmax, int rounding) {
  const int q = quant_code(t, inv, qmax, rounding);
  const double e = (double)t - (double)q * (double)scale;
  return e * e;
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int m = 1; m < 64; m *= 2) v += __shfl_xor(v, m);
  return v;
}

// One row per workgroup iteration; partial[2*row + {0,1}] = that row's sums.
template <int N>
__global__ __launch_bounds__(256) void quant_error_rows_kernel(
    const float* __restrict__ t, int64_t rows, int cols, int bits, int rounding,
    const float* __restrict__ rowmax, const float* __restrict__ partials, int npartials,
    double* __restrict__ partial) {
  __shared__ double s_sum[2][4];
  const int tid = threadIdx.x;
  const int qmax = (1 << (bits - 1)) - 1;
  const int nvec = cols / 4;
  const float amax_ten = block_max_of(partials, npartials);
  const float inv_ten = quant_inv(amax_ten, qmax), sc_ten = quant_scale(amax_ten, qmax);
  for (int64_t row = blockIdx.x; row < rows; row += gridDim.x) {
    const float4* src = reinterpret_cast<const float4*>(t + row * (int64_t)cols);
    const float amax_tok = rowmax[row];
    const float inv_tok = quant_inv(amax_tok, qmax), sc_tok = quant_scale(amax_tok, qmax);
    double e_tok = 0.0, e_ten = 0.0;
    for (int base = 0; base < nvec; base += 256) {  // uniform trip count keeps lanes converged
      const int i = base + tid;
      float4 q = i < nvec ? src[i] : make_float4(0.f, 0.f, 0.f, 0.f);
      fwht_row4<N>(q, tid);
      if (i < nvec) {
        e_tok += sq_err(q.x, inv_tok, sc_tok, qmax, rounding) + sq_err(q.y, inv_tok, sc_tok, qmax, rounding) +
                 sq_err(q.z, inv_tok, sc_tok, qmax, rounding) + sq_err(q.w, inv_tok, sc_tok, qmax, rounding);
        e_ten += sq_err(q.x, inv_ten, sc_ten, qmax, rounding) + sq_err(q.y, inv_ten, sc_ten, qmax, rounding) +
                 sq_err(q.z, inv_ten, sc_ten, qmax, rounding) + sq_err(q.w, inv_ten, sc_ten, qmax, rounding);
      }
    }
    e_tok = wave_sum(e_tok);
    e_ten = wave_sum(e_ten);
    if ((tid & 63) == 0) { s_sum[0][tid >> 6] = e_tok; s_sum[1][tid >> 6] = e_ten; }
    __syncthreads();
    if (tid == 0) {
      partial[2 * row + 0] = (s_sum[0][0] + s_sum[0][1]) + (s_sum[0][2] + s_sum[0][3]);
      partial[2 * row + 1] = (s_sum[1][0] + s_sum[1][1]) + (s_sum[1][2] + s_sum[1][3]);
    }
    __syncthreads();
  }
}

// Single workgroup: result[c] = sum over rows of partial[2*row + c], fixed order.
__global__ __launch_bounds__(256) void quant_error_final_kernel(const double* __restrict__ partial,
                                                                int64_t rows,
                                                                double* __restrict__ result) {
  __shared__ double s_sum[2][256];
  const int tid = threadIdx.x;
  double a = 0.0, b = 0.0;
  for (int64_t row = tid; row < rows; row += 256) { a += partial[2 * row]; b += partial[2 * row + 1]; }
  s_sum[0][tid] = a;
  s_sum[1][tid] = b;
  __syncthreads();
  for (int h = 128; h > 0; h >>= 1) {
    if (tid < h) { s_sum[0][tid] += s_sum[0][tid + h]; s_sum[1][tid] += s_sum[1][tid + h]; }
    __syncthreads();
  }
  if (tid == 0) { result[0] = s_sum[0][0]; result[1] = s_sum[1][0]; }
}

hipError_t launch_quant_error(const float* t, int64_t rows, int64_t cols, int n, int bits,
                              int rounding, const float* rowmax, const float* partials,
                              int npartials, double* partial, double* result, hipStream_t s) {
  const unsigned grid = (unsigned)(rows < 4096 ? rows : 4096);
  switch (n) {
    case 16: quant_error_rows_kernel<16><<<dim3(grid), dim3(256), 0, s>>>(t, rows, (int)cols, bits, rounding, rowmax, partials, npartials, partial); break;
    case 32: quant_error_rows_kernel<32><<<dim3(grid), dim3(256), 0, s>>>(t, rows, (int)cols, bits, rounding, rowmax, partials, npartials, partial); break;
    case 64: quant_error_rows_kernel<64><<<dim3(grid), dim3(256), 0, s>>>(t, rows, (int)cols, bits, rounding, rowmax, partials, npartials, partial); break;
    default: return hipErrorInvalidValue;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  quant_error_final_kernel<<<dim3(1), dim3(256), 0, s>>>(partial, rows, result);
  return hipGetLastError();
}

}  // namespace hot
