// Launcher of the fused g_y kernels (gy_fused_kernel.h).
#include "gy_fused_kernel.h"

namespace hot {

bool gy_fused_supported(const Config& c) { return c.n == 16 || c.n == 32; }

int64_t gy_fused_tiles_x(int64_t O) { return ceil_div(O, kFusedCT); }

namespace {

struct FusedArgs {
  const float* g;
  int64_t L, O;
  KeepMap map;
  int r, rounding;
  float *part_hla, *part_row, *rowpart;
  uint8_t* qg;
  int64_t pitch_g;
  float* sg;
  uint8_t* qgh;
  int64_t pitch_h;
  float* s_gh;
};

struct FusedPlan {
  int kbw_a, grid_a, kbw_q;
  int64_t tiles_q;
  size_t lds_q;
};

FusedPlan plan_fused(int64_t L, int64_t O, int n, int bpb) {
  FusedPlan p;
  const int64_t nblk = L / n, tiles_x = gy_fused_tiles_x(O);
  auto tiles = [&](int kbw) { return tiles_x * ceil_div(nblk, 4 * kbw); };
  p.kbw_a = 2;
  while (tiles(p.kbw_a) < 1024 && p.kbw_a > 1) p.kbw_a /= 2;
  const int64_t ta = tiles(p.kbw_a);
  p.grid_a = (int)(ta < kMaxPartials ? ta : kMaxPartials);
  // enough blocks per wave for 128-byte HLA runs per column
  p.kbw_q = 32 / bpb;
  p.kbw_q = p.kbw_q < 1 ? 1 : (p.kbw_q > 4 ? 4 : p.kbw_q);
  while (tiles(p.kbw_q) < 512 && p.kbw_q > 1) p.kbw_q /= 2;
  p.tiles_q = tiles(p.kbw_q);
  p.lds_q = (size_t)4 * p.kbw_q * n * 4 + (size_t)kFusedCT * (4 * p.kbw_q * bpb + 4);
  return p;
}

template <int N, int KIND, bool PER_TOKEN>
hipError_t launch_pass1(const FusedArgs& a, const FusedPlan& p, hipStream_t s) {
  gy_fused_absmax_kernel<N, KIND, PER_TOKEN><<<dim3((unsigned)p.grid_a), dim3(256), 0, s>>>(
      a.g, a.L, a.O, a.map, p.kbw_a, a.part_hla, a.part_row, a.rowpart);
  return hipGetLastError();
}

template <int N, int KIND, int BITS, bool PER_TOKEN, int ROUNDING>
hipError_t launch_pass2r(const FusedArgs& a, const FusedPlan& p, hipStream_t s) {
  gy_fused_quant_kernel<N, KIND, BITS, PER_TOKEN, ROUNDING><<<dim3((unsigned)p.tiles_q), dim3(256), p.lds_q, s>>>(
      a.g, a.L, a.O, a.map, a.r, p.kbw_q, a.part_hla, a.part_row, p.grid_a, a.rowpart,
      a.qg, a.pitch_g, a.sg, a.qgh, a.pitch_h, a.s_gh);
  return hipGetLastError();
}

template <int N, int KIND, int BITS, bool PER_TOKEN>
hipError_t launch_pass2(const FusedArgs& a, const FusedPlan& p, hipStream_t s) {
  return a.rounding == HOT_ROUND_NEAREST_EVEN ? launch_pass2r<N, KIND, BITS, PER_TOKEN, 0>(a, p, s)
                                              : launch_pass2r<N, KIND, BITS, PER_TOKEN, 1>(a, p, s);
}

template <int N, int KIND, bool PER_TOKEN>
hipError_t launch_both(const FusedArgs& a, const FusedPlan& p, int bits, hipStream_t s, int st1, int st2) {
  stage_begin(st1, s);
  hipError_t e = launch_pass1<N, KIND, PER_TOKEN>(a, p, s);
  stage_end(st1, s);
  if (e != hipSuccess) return e;
  stage_begin(st2, s);
  e = bits == 4 ? launch_pass2<N, KIND, 4, PER_TOKEN>(a, p, s) : launch_pass2<N, KIND, 8, PER_TOKEN>(a, p, s);
  stage_end(st2, s);
  return e;
}

template <int N>
hipError_t launch_n(const FusedArgs& a, const FusedPlan& p, int kind, bool per_token, int bits,
                    hipStream_t s, int st1, int st2) {
  if (kind == kKeepLowHalf)
    return per_token ? launch_both<N, kKeepLowHalf, true>(a, p, bits, s, st1, st2)
                     : launch_both<N, kKeepLowHalf, false>(a, p, bits, s, st1, st2);
  return per_token ? launch_both<N, kKeepGeneric, true>(a, p, bits, s, st1, st2)
                   : launch_both<N, kKeepGeneric, false>(a, p, bits, s, st1, st2);
}

}  // namespace

hipError_t launch_gy_fused(const float* g_y, int64_t L, int64_t O, const Config& cfg, bool per_token,
                           uint8_t* qg, int64_t pitch_g, float* sg, uint8_t* qgh, int64_t pitch_h,
                           float* s_gh, float* part_hla, float* part_row, float* rowpart,
                           hipStream_t s, int stage_absmax, int stage_quant) {
  if (!gy_fused_supported(cfg) || L <= 0 || O <= 0 || L % cfg.n || O % cfg.n) return hipErrorInvalidValue;
  const int kind = (cfg.lowpass_default && cfg.r * 2 == cfg.n) ? kKeepLowHalf : kKeepGeneric;
  const FusedPlan p = plan_fused(L, O, cfg.n, cfg.r);
  const FusedArgs a{g_y, L, O, cfg.map, cfg.r, cfg.rounding, part_hla, part_row, rowpart,
                    qg, pitch_g, sg, qgh, pitch_h, s_gh};
  if (cfg.n == 16) return launch_n<16>(a, p, kind, per_token, cfg.gx_bits, s, stage_absmax, stage_quant);
  return launch_n<32>(a, p, kind, per_token, cfg.gx_bits, s, stage_absmax, stage_quant);
}

}  // namespace hot
