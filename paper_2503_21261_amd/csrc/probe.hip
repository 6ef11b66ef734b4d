// Machine-peak probes for the benchmark's context figures: a plain HBM read, a
// plain HBM write, and a register-only int8 matrix-core loop.  Not on any hot path.
#include "hot_host.h"

namespace hot {

typedef int pv4i __attribute__((ext_vector_type(4)));
typedef int pv16i __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void probe_read_kernel(const float4* __restrict__ p, size_t n,
                                                         float* __restrict__ sink) {
  float s = 0.0f;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    const float4 v = p[i];
    s += v.x + v.y + v.z + v.w;
  }
  if (s == 1.2345678f) sink[0] = s;  // keeps the loads alive; practically never true
}

__global__ __launch_bounds__(256) void probe_write_kernel(float4* __restrict__ p, size_t n, float v) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256)
    p[i] = make_float4(v, v, v, v);
}

// The same with the streaming (non-temporal) hint the GEMM epilogue uses.
typedef float pv4f __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void probe_write_nt_kernel(pv4f* __restrict__ p, size_t n, float v) {
  const pv4f q = {v, v, v, v};
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256)
    __builtin_nontemporal_store(q, &p[i]);
}

// 16 independent 32x32 accumulators per wave, operands in registers.
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, int random_operands,
                                                         int* __restrict__ sink) {
  pv4i a = {(int)threadIdx.x, 1, 2, 3}, b = {4, 5, 6, (int)threadIdx.x};
  if (random_operands) {
    unsigned x = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
    for (int i = 0; i < 4; ++i) {
      x ^= x >> 13; x *= 0x5bd1e995u; x ^= x >> 15; a[i] = (int)x;
      x *= 0x846ca68bu; x ^= x >> 16; b[i] = (int)x;
    }
  }
  pv16i acc[16];
  for (int i = 0; i < 16; ++i)
    for (int v = 0; v < 16; ++v) acc[i][v] = 0;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[i], 0, 0, 0);
  }
  int s = 0;
  for (int i = 0; i < 16; ++i)
    for (int v = 0; v < 16; ++v) s += acc[i][v];
  sink[blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace hot

extern "C" hot_status hot_debug_probe(int kind, void* buf, size_t bytes, int iters, void* stream) {
  using namespace hot;
  if (!buf || bytes < (1u << 20) || iters < 1) return HOT_ERR_ARG;
  hipStream_t s = (hipStream_t)stream;
  const size_t n4 = (bytes - 4096) / 16;
  switch (kind) {
    case 0: probe_read_kernel<<<dim3(4096), dim3(256), 0, s>>>((const float4*)buf, n4, (float*)buf + n4 * 4); break;
    case 1: probe_write_kernel<<<dim3(4096), dim3(256), 0, s>>>((float4*)buf, n4, 1.0f); break;
    case 2:
    case 3: probe_mfma_kernel<<<dim3(256), dim3(256), 0, s>>>(iters, kind == 3, (int*)buf); break;
    case 4: probe_write_nt_kernel<<<dim3(4096), dim3(256), 0, s>>>((pv4f*)buf, n4, 1.0f); break;
    default: return HOT_ERR_ARG;
  }
  return hipGetLastError() == hipSuccess ? HOT_OK : HOT_ERR_DEVICE;
}
