// First launch of the g_x path (Sec. 5.1) when both of its operands are produced in one
// kernel: the leading workgroups transform and quantise the weights (H.w, one scale, the
// single-pass column kernel with its abs-max exchange), the rest rotate and quantise the
// rows of g_y per token.  The two jobs are independent; sharing a launch lets the rows
// stream from HBM while the few weight workgroups sit in the latencies of their exchange,
// which as a kernel of its own is 13 us of a mostly idle chip for the ViT-B weights.
#include <mutex>

#include "col_quant_kernel.h"
#include "row_quant_kernel.h"

namespace hot {

namespace {

template <int N, int KB, int ITER, int TPR>
__global__ __launch_bounds__(256, 2) void w_and_rows_kernel(const OnepassArgs wa, const int w_tiles,
                                                            const RowQuantArgs ra) {
  // workgroups are dispatched in index order: the weight tiles, which must all be resident
  // for their exchange to complete without the fallback, come first
  if ((int)blockIdx.x < w_tiles)
    onepass_body<N, onepass_vec(N), kKeepAll4, KB>(wa, (int)blockIdx.x, w_tiles);
  else
    row_quant_body<N, ITER, TPR>(ra, (int64_t)blockIdx.x - w_tiles, (int64_t)gridDim.x - w_tiles);
}

struct FrontArgs {
  OnepassArgs wa;
  RowQuantArgs ra;
  int64_t nrb;   // row workgroups
};

template <int N, int KB, int ITER, int TPR>
hipError_t try_front(const FrontArgs& f, hipStream_t s, int stage, bool* done) {
  constexpr int VEC = onepass_vec(N);
  if (*done || f.wa.C % VEC != 0) return hipSuccess;
  const int64_t tiles = ceil_div(f.wa.C, 64 * VEC) * ceil_div(f.wa.rt.nblk, 4 * KB);
  size_t lds = (size_t)(64 * VEC) * (4 * KB * (N / 2) + 4);
  if (lds < onepass_stage_bytes<N, VEC, kKeepAll4>()) lds = onepass_stage_bytes<N, VEC, kKeepAll4>();
  auto kern = w_and_rows_kernel<N, KB, ITER, TPR>;
  static std::mutex mu;
  static int per_cu = -1, cus = 0;
  {
    std::lock_guard<std::mutex> lock(mu);
    if (per_cu < 0) {
      int dev = 0, nb = 0;
      hipError_t e = hipGetDevice(&dev);
      if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
      if (e == hipSuccess && lds > 48 * 1024)
        e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, kern, 256, lds);
      if (e != hipSuccess) return e;
      per_cu = nb;
    }
  }
  if (tiles > (int64_t)per_cu * cus || tiles > kMaxExchange) return hipSuccess;
  stage_begin(stage, s);
  kern<<<dim3((unsigned)(tiles + f.nrb)), dim3(256), lds, s>>>(f.wa, (int)tiles, f.ra);
  stage_end(stage, s);
  *done = true;
  return hipGetLastError();
}

template <int N, int ITER, int TPR>
hipError_t front_kb(const FrontArgs& f, hipStream_t s, int stage, bool* done) {
  hipError_t e = try_front<N, 1, ITER, TPR>(f, s, stage, done);
  if (e == hipSuccess && !*done) e = try_front<N, 2, ITER, TPR>(f, s, stage, done);
  return e;
}

template <int N>
hipError_t front_n(FrontArgs& f, hipStream_t s, int stage, bool* done) {
  const int cols = f.ra.cols;
  const int v64 = (int)ceil_div(cols, 256), v256 = (int)ceil_div(cols, 1024);
  // the row kernel's own choice of threads per row and values per thread (row_quant.hip)
  if (v64 <= 1) return hipSuccess;
  if (v64 <= 4) f.nrb = ceil_div(f.ra.rows, 4);
  else f.nrb = f.ra.rows;
  if (f.nrb > (1 << 20)) return hipSuccess;
  if (v64 == 2) return front_kb<N, 2, 64>(f, s, stage, done);
  if (v64 == 3) return front_kb<N, 3, 64>(f, s, stage, done);
  if (v64 == 4) return front_kb<N, 4, 64>(f, s, stage, done);
  if (v256 == 2) return front_kb<N, 2, 256>(f, s, stage, done);
  if (v256 == 3) return front_kb<N, 3, 256>(f, s, stage, done);
  if (v256 == 4) return front_kb<N, 4, 256>(f, s, stage, done);
  return hipSuccess;
}

}  // namespace

hipError_t launch_w_and_rows(const float* w, int64_t O, int64_t I, const Config& cfg, uint8_t* qw,
                             int64_t pitch, float* s_w, float* slots, const float* g_y, int64_t L,
                             uint8_t* qg, float* s_g, hipStream_t s, int stage, bool* done) {
  *done = false;
  int64_t wait_us = exchange_wait_us();
  if (wait_us < 0 || cfg.gx_bits != 4 || O % cfg.n != 0 || L <= 0 || I <= 0) return hipSuccess;
  const int64_t stream_us = O * I * 4 / 1000000;   // as in the column kernel's own launcher
  if (wait_us > 0 && wait_us < stream_us) wait_us = stream_us;
  KeepMap id;
  for (int k = 0; k < 64; ++k) id.pos[k] = (int8_t)(k < cfg.n ? k : -1);
  FrontArgs f;
  f.wa = OnepassArgs{w, RowTiling{O / cfg.n, 0, 1}, I, id, cfg.n, cfg.rounding,
                     reinterpret_cast<unsigned long long*>(slots), next_exchange_tag(), cfg.epoch,
                     (long long)(wait_us * 100), qw, pitch, s_w};
  f.ra = RowQuantArgs{g_y, L, (int)O, 4, cfg.rounding, 0, qg, pitch, s_g, nullptr, 0};
  f.nrb = 0;
  switch (cfg.n) {
    case 16: return front_n<16>(f, s, stage, done);
    case 32: return front_n<32>(f, s, stage, done);
    case 64: return front_n<64>(f, s, stage, done);
  }
  return hipSuccess;
}

}  // namespace hot
