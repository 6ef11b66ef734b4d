// Launchers of the row-direction transform/quantise kernels (row_quant_kernel.h) and the
// streamed variant for rows too long for registers.
#include "hot_host.h"
#include "row_quant_kernel.h"

namespace hot {

// Rows longer than the register-resident variants cover: one row per workgroup,
// transformed twice (abs-max pass, then quantise pass; the second read hits L2).
template <int N>
__global__ __launch_bounds__(256) void row_quant_stream_kernel(
    const float* __restrict__ t, int64_t rows, int cols, int bits, int rounding, int mode,
    uint8_t* __restrict__ codes, int64_t pitch, float* __restrict__ scales,
    float* __restrict__ partials, int npartials) {
  __shared__ float s_max[4];
  const int tid = threadIdx.x;
  const int qmax = (1 << (bits - 1)) - 1;
  const int valid_bytes = cols * bits / 8;
  const int nvec = cols / 4;
  float running = 0.0f;
  float amax_tensor = 0.0f;
  if (mode == 2) amax_tensor = block_max_of(partials, npartials);
  for (int64_t row = blockIdx.x; row < rows; row += gridDim.x) {
    const float4* src = reinterpret_cast<const float4*>(t + row * (int64_t)cols);
    float amax;
    if (mode == 2) {
      amax = amax_tensor;
    } else {
      float m = 0.0f;
      for (int base = 0; base < nvec; base += 256) {  // uniform trip count: shuffles stay converged
        const int i = base + tid;
        float4 q = i < nvec ? src[i] : make_float4(0.f, 0.f, 0.f, 0.f);
        fwht_row4<N>(q, tid);
        m = fmaxf(m, absmax4(q));
      }
      m = wave_max(m);
      if ((tid & 63) == 0) s_max[tid >> 6] = m;
      __syncthreads();
      amax = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));
      __syncthreads();
    }
    if (mode == 1 || mode == 3) {
      running = fmaxf(running, amax);
      if (mode == 3 && tid == 0) scales[row] = amax;
      continue;
    }
    if (mode == 0 && tid == 0) scales[row] = quant_scale(amax, qmax);
    const float inv = quant_inv(amax, qmax);
    uint8_t* row_codes = codes + row * pitch;
    for (int base = 0; base < nvec; base += 256) {
      const int i = base + tid;
      float4 q = i < nvec ? src[i] : make_float4(0.f, 0.f, 0.f, 0.f);
      fwht_row4<N>(q, tid);
      if (i < nvec) store_codes4(row_codes, i * 4, q, inv, qmax, bits, rounding);
    }
    for (int off = valid_bytes + 4 * tid; off < pitch; off += 4 * 256)
      *reinterpret_cast<uint32_t*>(row_codes + off) = 0u;
  }
  if (mode == 1 || mode == 3) {
    if (tid == 0) partials[blockIdx.x] = running;
  } else if (mode == 2 && blockIdx.x == 0 && tid == 0) {
    scales[0] = quant_scale(amax_tensor, qmax);
  }
}

namespace {

constexpr int kMaxGrid = kMaxPartials;  // abs-max modes: one partial maximum per workgroup

template <int N>
hipError_t dispatch_row_quant(const float* t, int64_t rows, int cols, int bits, int rounding,
                              int mode, uint8_t* codes, int64_t pitch, float* scales,
                              float* partials, int* npartials, hipStream_t s) {
#define HOT_LAUNCH(ITER, TPR)                                                                  \
  {                                                                                            \
    const int64_t nrb = ceil_div(rows, 256 / TPR);                                             \
    const unsigned grid = (unsigned)((mode == 1 || mode == 3) ? (nrb < kMaxGrid ? nrb : kMaxGrid) \
                                                              : (nrb < (1 << 20) ? nrb : (1 << 20))); \
    if (mode == 1 || mode == 3) *npartials = (int)grid;                                        \
    const RowQuantArgs ra{t, rows, cols, bits, rounding, mode, codes, pitch, scales, partials,  \
                          *npartials};                                                        \
    row_quant_kernel<N, ITER, TPR><<<dim3(grid), dim3(256), 0, s>>>(ra);                       \
    return hipGetLastError();                                                                  \
  }
  const int v64 = (int)ceil_div(cols, 256);    // float4 per thread with one wave per row
  const int v256 = (int)ceil_div(cols, 1024);  // float4 per thread with one workgroup per row
  if (v64 <= 1) HOT_LAUNCH(1, 64)
  if (v64 <= 2) HOT_LAUNCH(2, 64)
  if (v64 <= 3) HOT_LAUNCH(3, 64)
  if (v64 <= 4) HOT_LAUNCH(4, 64)
  if (v256 <= 2) HOT_LAUNCH(2, 256)
  if (v256 <= 3) HOT_LAUNCH(3, 256)
  if (v256 <= 4) HOT_LAUNCH(4, 256)
  if (v256 <= 6) HOT_LAUNCH(6, 256)
  if (v256 <= 8) HOT_LAUNCH(8, 256)
  if (v256 <= 11) HOT_LAUNCH(11, 256)
  if (v256 <= 16) HOT_LAUNCH(16, 256)
#undef HOT_LAUNCH
  const unsigned grid = (unsigned)(rows < kMaxGrid ? rows : kMaxGrid);
  if (mode == 1 || mode == 3) *npartials = (int)grid;
  row_quant_stream_kernel<N><<<dim3(grid), dim3(256), 0, s>>>(t, rows, cols, bits, rounding, mode,
                                                              codes, pitch, scales, partials, *npartials);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_row_quant(const float* t, int64_t rows, int64_t cols, int n, int bits,
                            int rounding, int mode, uint8_t* codes, int64_t pitch, float* scales,
                            float* partials, int* npartials, hipStream_t s) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  switch (n) {
    case 16: return dispatch_row_quant<16>(t, rows, (int)cols, bits, rounding, mode, codes, pitch, scales, partials, npartials, s);
    case 32: return dispatch_row_quant<32>(t, rows, (int)cols, bits, rounding, mode, codes, pitch, scales, partials, npartials, s);
    case 64: return dispatch_row_quant<64>(t, rows, (int)cols, bits, rounding, mode, codes, pitch, scales, partials, npartials, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace hot
