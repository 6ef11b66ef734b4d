// Launch plan and launcher of the column-direction transform/quantise kernels
// (col_quant_kernel.h).
#include <atomic>
#include <chrono>
#include <mutex>

#include "col_quant_kernel.h"

namespace hot {

namespace {
// Microseconds a single-pass workgroup waits for the other workgroups' maxima before it
// computes the missing ones itself; < 0 disables the single-pass kernels.
std::atomic<int> g_exchange_wait_us{200};

// Launch tags: 64 bits that never repeat within a process (a counter) and differ between
// processes (it starts at the clock's nanosecond count), so that a slot or flag left in a
// workspace by any earlier launch, of this process or another, is never taken for a fresh one:
// a leftover would have to match all 64 bits.
uint64_t next_tag() {
  static std::atomic<uint64_t> tag{(uint64_t)std::chrono::steady_clock::now().time_since_epoch().count() | 1u};
  uint64_t t = tag.fetch_add(1, std::memory_order_relaxed);
  return t ? t : tag.fetch_add(1, std::memory_order_relaxed);   // zero is never a tag
}
}  // namespace

void set_exchange_wait_us(int us) { g_exchange_wait_us.store(us); }
int exchange_wait_us() { return g_exchange_wait_us.load(); }
uint64_t next_exchange_tag() { return next_tag(); }

ColPlan plan_col(int64_t nblk, int64_t C, int n, int r, int bits, bool lowpass_default, bool identity) {
  ColPlan p;
  if (bits == 4) p.kind = kKeepAll4;
  else if (identity && r == n) p.kind = kKeepAll8;
  else if (lowpass_default && r * 2 == n) p.kind = kKeepLowHalf;
  else p.kind = kKeepGeneric;
  const int bpb = bits == 4 ? n / 2 : r;
  const int vdiv = (C % 4 == 0) ? 4 : (C % 2 == 0 ? 2 : 1);
  auto tiles = [&](int vec, int kbw) { return ceil_div(C, 64 * vec) * ceil_div(nblk, 4 * kbw); };
  // Abs-max pass (a workgroup tile is 256 * vec columns x kbw blocks): about 64 rows per
  // wave and visit, two columns per lane (measured on MI355X for 16-row blocks: 556 us with
  // two against 580-596 us with four on 3.3 GB, 119 against 123 us on 620 MB, one column
  // 124 us); smaller tiles while the 256 compute units would otherwise be short of
  // workgroups, narrower ones for narrow tensors.
  auto tiles_a = [&](int vec, int kbw) { return ceil_div(C, 256 * vec) * ceil_div(nblk, kbw); };
  const int vpref = 2;
  p.vec_a = vdiv < vpref ? vdiv : vpref;
  while (p.vec_a > 1 && C < 256 * p.vec_a) p.vec_a /= 2;
  p.kbw_a = n >= 64 ? 1 : 64 / n;
  while (tiles_a(p.vec_a, p.kbw_a) < 1024 && p.kbw_a > 1) p.kbw_a /= 2;
  while (tiles_a(p.vec_a, p.kbw_a) < 512 && p.vec_a > 1) p.vec_a /= 2;
  const int64_t ta = tiles_a(p.vec_a, p.kbw_a);
  p.absmax_grid = (int)(ta < kMaxPartials ? ta : kMaxPartials);
  // Quantise pass: measured fastest with one column per lane (few registers, many
  // waves) and enough blocks per wave for 256-byte output runs per column.
  p.vec_q = 1;
  p.kbw_q = 64 / bpb;
  p.kbw_q = p.kbw_q < 1 ? 1 : (p.kbw_q > 8 ? 8 : p.kbw_q);
  while (tiles(p.vec_q, p.kbw_q) < 512 && p.kbw_q > 1) p.kbw_q /= 2;
  p.tiles_q = tiles(p.vec_q, p.kbw_q);
  p.lds_q = (size_t)(64 * p.vec_q) * (4 * p.kbw_q * bpb + 4);
  return p;
}

namespace {

struct ColArgs {
  const float* x;
  RowTiling rows;
  int64_t C;
  KeepMap map;
  int r, rounding;
  uint8_t* codes;
  int64_t pitch;
  float* scale;
  float* partials;
  const unsigned long long* epoch;
};

template <int N, int VEC, int KIND>
hipError_t launch_absmax(const ColArgs& a, const ColPlan& p, hipStream_t s) {
  col_absmax_kernel<N, VEC, KIND><<<dim3((unsigned)p.absmax_grid), dim3(256), 0, s>>>(
      a.x, a.rows, a.C, a.map, p.kbw_a, a.partials);
  return hipGetLastError();
}

template <int N, int VEC, int KIND>
hipError_t launch_quant(const ColArgs& a, const ColPlan& p, hipStream_t s) {
  col_quant_kernel<N, VEC, KIND><<<dim3((unsigned)p.tiles_q), dim3(256), p.lds_q, s>>>(
      a.x, a.rows, a.C, a.map, a.r, a.rounding, p.kbw_q, a.partials, p.absmax_grid, a.codes, a.pitch,
      a.scale);
  return hipGetLastError();
}

// Single-pass launch with KB blocks per wave; *done stays false (nothing launched) when
// that grid would not be resident all at once or the lane would hold too many values.
template <int N, int KIND, int KB>
hipError_t try_onepass(const ColArgs& a, hipStream_t s, int sq, int round, bool* done) {
  constexpr int VEC = onepass_vec(N);
  if constexpr (onepass_kept_regs<N, VEC, KIND, KB>() > kOnepassMaxKept) {
    return hipSuccess;
  } else {
    if (*done || a.C % VEC != 0) return hipSuccess;
    const int bpb = KIND == kKeepGeneric ? a.r : (KIND == kKeepAll8 ? N : N / 2);
    const int64_t tiles = ceil_div(a.C, 64 * VEC) * ceil_div(a.rows.nblk, 4 * KB);
    // rounds 0 and 1: only launch shapes whose lanes store their codes straight from
    // registers (round 0: in runs that fill whole 128-byte lines per workgroup) and that
    // still give every compute unit more than one workgroup
    const bool direct_only = round < 2;
    if (direct_only && !onepass_direct_store<N, KIND, KB>()) return hipSuccess;
    if (round == 0 && !onepass_whole_lines<N, KIND, KB>()) return hipSuccess;
    size_t lds = (size_t)(64 * VEC) * (4 * KB * bpb + 4);
    if (lds < onepass_stage_bytes<N, VEC, KIND>()) lds = onepass_stage_bytes<N, VEC, KIND>();
    auto kern = col_quant_onepass_kernel<N, VEC, KIND, KB>;
    constexpr size_t lds_tile_max = (size_t)(64 * VEC) * (4 * KB * N + 4);   // bpb <= N
    constexpr size_t lds_max = lds_tile_max > onepass_stage_bytes<N, VEC, KIND>()
                                   ? lds_tile_max : onepass_stage_bytes<N, VEC, KIND>();
    static std::mutex mu;              // per instantiation: the cached occupancy below
    static int per_cu = -1, cus = 0;   // for the LDS size last asked for
    static size_t lds_seen = 0;
    std::lock_guard<std::mutex> lock(mu);
    if (per_cu < 0 || lds != lds_seen) {
      int dev = 0, nb = 0;
      hipError_t e = hipGetDevice(&dev);
      if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
      if (e == hipSuccess && per_cu < 0 && lds_max > 48 * 1024)
        e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_max);
      if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, kern, 256, lds);
      if (e != hipSuccess) return e;
      per_cu = nb;
      lds_seen = lds;
    }
    if (tiles > (int64_t)per_cu * cus || tiles > kMaxExchange) return hipSuccess;
    if (direct_only && tiles * 4 < 5 * (int64_t)cus) return hipSuccess;
    // ... and at most two: with three or more per compute unit both the read and the final
    // stores measured slower (155 MB of 16-row blocks: 48.7 us on 678 workgroups of 7 blocks
    // per wave against 41.1 us on 474 of 10)
    if (direct_only && tiles > 2 * (int64_t)cus) return hipSuccess;
    // the other workgroups need at least the time to stream their share of the input:
    // never wait less than the whole tensor takes at 1 TB/s (0 stays 0: tests force the
    // self-computed path with it)
    int64_t wait_us = g_exchange_wait_us.load();
    const int64_t stream_us = a.rows.nblk * N * a.C * 4 / 1000000;
    if (wait_us > 0 && wait_us < stream_us) wait_us = stream_us;
    stage_begin(sq, s);
    const OnepassArgs oa{a.x, a.rows, a.C, a.map, a.r, a.rounding,
                         reinterpret_cast<unsigned long long*>(a.partials), next_tag(), a.epoch,
                         (long long)(wait_us * 100), a.codes, a.pitch, a.scale};
    kern<<<dim3((unsigned)tiles), dim3(256), lds, s>>>(oa);
    stage_end(sq, s);
    *done = true;
    return hipGetLastError();
  }
}

// The smallest number of blocks per wave (most workgroups, most loads in flight) whose grid
// is resident at once; none fits a tensor whose kept values exceed the register files.
// A shape whose lanes hold enough consecutive output bytes to store them directly (no
// pass through the LDS tile after the exchange, measured 2 us shorter on the ViT-B
// activations) is preferred while it leaves between 1.25 and 2 workgroups per compute unit, and
// among those one whose workgroups write whole 128-byte lines of every output row, so that no
// line is shared with a workgroup on another XCD (HLA of the ViT-B g_y: 43.1 us with 10
// blocks per wave against 44.8 us with 7).
template <int N, int KIND>
hipError_t launch_onepass(const ColArgs& a, hipStream_t s, int sq, bool* done) {
  hipError_t e = hipSuccess;
#define HOT_TRY_KB(KB, ROUND) \
  if (e == hipSuccess && !*done) e = try_onepass<N, KIND, KB>(a, s, sq, ROUND, done);
  HOT_TRY_KB(1, 0) HOT_TRY_KB(2, 0) HOT_TRY_KB(4, 0) HOT_TRY_KB(8, 0) HOT_TRY_KB(10, 0)
  HOT_TRY_KB(1, 1) HOT_TRY_KB(2, 1) HOT_TRY_KB(3, 1) HOT_TRY_KB(4, 1) HOT_TRY_KB(5, 1) HOT_TRY_KB(7, 1)
  HOT_TRY_KB(8, 1) HOT_TRY_KB(10, 1)
  HOT_TRY_KB(1, 2) HOT_TRY_KB(2, 2) HOT_TRY_KB(3, 2) HOT_TRY_KB(4, 2) HOT_TRY_KB(5, 2) HOT_TRY_KB(7, 2)
  HOT_TRY_KB(8, 2) HOT_TRY_KB(10, 2)
#undef HOT_TRY_KB
  return e;
}

template <int N, int KIND>
hipError_t launch_nk(const ColArgs& a, const ColPlan& p, hipStream_t s, int sa, int sq) {
  if (g_exchange_wait_us.load() >= 0) {
    bool done = false;
    const hipError_t e1 = launch_onepass<N, KIND>(a, s, sq, &done);
    if (e1 != hipSuccess || done) return e1;
  }
  hipError_t e = hipErrorInvalidValue;
  stage_begin(sa, s);
  if constexpr (N < 64) {
    if (p.vec_a == 4) e = launch_absmax<N, 4, KIND>(a, p, s);
  }
  if (p.vec_a == 2) e = launch_absmax<N, 2, KIND>(a, p, s);
  if (p.vec_a == 1) e = launch_absmax<N, 1, KIND>(a, p, s);
  stage_end(sa, s);
  if (e != hipSuccess) return e;
  stage_begin(sq, s);
  e = launch_quant<N, 1, KIND>(a, p, s);
  stage_end(sq, s);
  return e;
}

template <int N>
hipError_t launch_n(const ColArgs& a, const ColPlan& p, hipStream_t s, int sa, int sq) {
  switch (p.kind) {
    case kKeepLowHalf: return launch_nk<N, kKeepLowHalf>(a, p, s, sa, sq);
    case kKeepAll8: return launch_nk<N, kKeepAll8>(a, p, s, sa, sq);
    case kKeepAll4: return launch_nk<N, kKeepAll4>(a, p, s, sa, sq);
    default: return launch_nk<N, kKeepGeneric>(a, p, s, sa, sq);
  }
}

}  // namespace

hipError_t launch_col_quant(const float* x, const RowTiling& rows, int64_t C, const Config& cfg, int r,
                            const KeepMap& map, bool identity, int bits, uint8_t* codes,
                            int64_t pitch, float* scale, float* partials, hipStream_t s,
                            int stage_absmax, int stage_quant) {
  if (rows.nblk <= 0 || C <= 0) return hipSuccess;
  if (bits == 4 && !(identity && r == cfg.n)) return hipErrorInvalidValue;
  const ColPlan p = plan_col(rows.nblk, C, cfg.n, r, bits, cfg.lowpass_default && !identity, identity);
  const ColArgs a{x, rows, C, map, r, cfg.rounding, codes, pitch, scale, partials, cfg.epoch};
  switch (cfg.n) {
    case 16: return launch_n<16>(a, p, s, stage_absmax, stage_quant);
    case 32: return launch_n<32>(a, p, s, stage_absmax, stage_quant);
    case 64: return launch_n<64>(a, p, s, stage_absmax, stage_quant);
  }
  return hipErrorInvalidValue;
}

}  // namespace hot
