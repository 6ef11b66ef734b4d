// Integer GEMM kernel on the CDNA4 matrix cores with fused dequantisation:
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
#pragma once
#include <type_traits>
#include <utility>

#include "hot_device.h"

namespace hot {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

// Compile-time loop: f(std::integral_constant<int, 0>) ... f(integral_constant<int, N-1>).
template <int... Is, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, Is...>, F&& f) {
  (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(std::make_integer_sequence<int, N>{}, static_cast<F&&>(f));
}

// One fp32 store with the streaming (non-temporal) cache hint, OFF bytes past p.
template <int OFF>
__device__ __forceinline__ void store_streaming(float* p, float v) {
  asm volatile("global_store_dword %0, %1, off offset:%2 nt" : : "v"(p), "v"(v), "n"(OFF) : "memory");
}

struct GemmArgs {
  const uint8_t* A;
  const uint8_t* B;
  int M, N;
  int nk_total;          // K stages of BKB bytes in the whole K range
  int64_t pitch;         // bytes per operand row
  int tiles_m, tiles_n;
  int32_t* out_i32;      // raw accumulators [M][N], or
  float* out_f32;        // dequantised output [M][N]
  // Split-K launches only (slot = tile * (split - 1) + slice, for all slices but the last):
  int split;                   // K slices
  int32_t* partial;            // [slot][register image of the 256-thread tile]
  unsigned long long* flags;   // [slot] = tag once the image is complete
  unsigned long long tag;      // 64 bits, never zero, never repeated: slots never need clearing
  const unsigned long long* epoch;   // replayable calls: the tag is moved by *epoch
  long long wait_ticks;        // bound on the wait for another workgroup's image (100 MHz ticks)
  const float* row_scale;
  int row_stride;
  const float* col_scale;
  float inv_n;
  int stream_out;        // fp32 output with non-temporal stores
  int xcd_cols;          // split-K: > 0: the tile grid cut into 8 / xcd_cols x xcd_cols rectangles, one per XCD;
                         // < 0: XCDs dealt to the K slices; 0: band walk
};

// Workgroup id -> output tile.  Workgroups are dealt round-robin to the 8 XCDs, each
// with its own L2: ids are regrouped so that one XCD walks a contiguous run of tiles,
// and a run is ordered in bands of kGroupM tile rows, tile row fastest inside a band.
// The ~32-96 workgroups resident on an XCD then cover kGroupM A tiles x a few B tiles,
// so every operand tile fetched over the fabric is reused from L2 by its neighbours
// (measured before this ordering: the A operand of the g_x GEMM was fetched once per
// tile column, 6x its size).
constexpr int kGroupM = 8;
__device__ __forceinline__ int xcd_contiguous(int id, int total) {
  const int per_xcd = total / 8;
  return id < per_xcd * 8 ? (id % 8) * per_xcd + id / 8 : id;
}
__device__ __forceinline__ void tile_of_position(const GemmArgs& g, int id, int& tm, int& tn) {
  const int band = kGroupM * g.tiles_n;
  const int first_m = (id / band) * kGroupM;
  int rows = g.tiles_m - first_m;
  rows = rows < kGroupM ? rows : kGroupM;
  const int in_band = id % band;
  tm = first_m + in_band % rows;
  tn = in_band / rows;
}

// ---- main loop ---------------------------------------------------------------------
// One wave per SIMD at the large INT4 tile (the accumulators of a 128x128 wave tile fill
// the AGPRs), two at the large INT8 tile (eight waves of 64x128), so latency is hidden inside
// the wave rather than by occupancy:
//   - global loads run two K stages ahead (registers), LDS holds two stages;
//   - the 16-byte LDS fragments of K slice ks+1 are read, and (INT4) widened, while
//     the matrix instructions of slice ks execute;
//   - one barrier per stage, placed before the last slice, so the first fragments
//     of the next stage are fetched under the last slice's matrix instructions;
//   - the loop is branch-free (tail iterations re-load and re-store a valid stage),
//     and every memory or widening instruction is pinned between two matrix
//     instructions so the matrix pipe never drains while the wave issues them.
template <int TM, int TN, bool INT4>
struct Operands {            // what the matrix instructions of one K slice consume
  v4i a[INT4 ? 2 : 1][TM];   // [low nibbles | high nibbles] or the int8 codes
  v4i b[INT4 ? 2 : 1][TN];
};

// BF16 = true: the same data movement with bfloat16 operands (16 bytes per lane are 8
// elements of v_mfma_f32_32x32x16_bf16) and fp32 accumulators; the "integer" outputs then
// carry the accumulators' fp32 bit patterns.
//
// SPLITK = false: workgroup b computes output tile b over the whole K range.
// SPLITK = true: the K range is cut into g.split slices and the grid holds one workgroup
// per (slice, tile), slice-major, so that workgroups running side by side work on
// neighbouring tiles at the same K offsets and share operand tiles through L2 exactly as
// without the split.  The workgroup of a tile's last slice owns the tile and writes its
// output; the others leave their accumulators as a register image in `partial` and announce
// it in `flags`.  Owners are dispatched last, so they normally find the images waiting.
// The wait is bounded: an owner that does not see an image in time computes that slice
// itself (integer sums do not depend on who adds what), so the kernel finishes even if
// workgroups are not resident together.
// Waves per SIMD the register allocation must leave room for: two for the 128x256 INT4 tile
// (its workgroups come in pairs per compute unit so that one's output stores run under the
// other's matrix instructions), whatever fits otherwise.
template <int BM, int BN, bool INT4>
constexpr int gemm_min_waves_per_simd() { return (INT4 && BM == 128 && BN == 256) ? 2 : 1; }

template <int BM, int BN, int WAVES_M, int WAVES_N, int BKB, bool INT4, bool BF16 = false,
          bool SPLITK = false>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N, (gemm_min_waves_per_simd<BM, BN, INT4>()))
void igemm_kernel(const GemmArgs g) {
  static_assert(!(INT4 && BF16), "one operand format");
  static_assert(!(SPLITK && BF16), "fp32 sums would depend on which workgroup added a piece");
  using acc_t = std::conditional_t<BF16, v16f, v16i>;
  constexpr int NT = 64 * WAVES_M * WAVES_N;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int LP = BKB;               // LDS row pitch; 16-byte chunks are XOR-swizzled (below)
  constexpr int TPR = BKB / 16;
  constexpr int RPP = NT / TPR;
  constexpr int PA = BM / RPP, PB = BN / RPP;
  constexpr int KS = BKB / 32;
  static_assert(BM % RPP == 0 && BN % RPP == 0, "loader passes");
  static_assert(KS >= 2 && KS % 2 == 0, "pipeline needs an even number of K slices per stage");
  extern __shared__ __align__(16) uint8_t smem[];
  __shared__ __align__(16) float s_rowfac[BM];   // row_scale[m] * col_scale / n for the rows of this tile
  __shared__ int s_seen;           // split-K: outcome of the wait for another workgroup's image
  uint8_t* As = smem;
  uint8_t* Bs = smem + 2 * BM * LP;

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wm0 = (wave % WAVES_M) * WM, wn0 = (wave / WAVES_M) * WN;

  // LDS layout: row r of a tile holds its BKB bytes as 16-byte chunks, chunk c stored at
  // position c ^ f(r), f(r) = (r >> 1) & 3 for 64-byte rows, r & 7 for 128-byte rows.  Any
  // 8 consecutive rows reading the same chunk, and any row writing its chunks, then hit 32
  // distinct banks: no padding, no conflicts.  f only uses row bits 0-2, so tile-row offsets
  // that are multiples of 8 keep a thread's swizzle constant.
  auto swz = [](int r) { return TPR == 4 ? (r >> 1) & 3 : r & 7; };
  const int lr = tid / TPR, lseg = (tid % TPR) * 16;
  const int st_off = lr * LP + 16 * ((tid % TPR) ^ swz(lr));
  int m0 = 0, n0 = 0;
  const uint8_t* a_src[PA];
  const uint8_t* b_src[PB];
  auto set_tile = [&](int tm, int tn) {
    m0 = tm * BM;
    n0 = tn * BN;
#pragma unroll
    for (int p = 0; p < PA; ++p) {
      int row = m0 + lr + RPP * p;
      row = row < g.M ? row : g.M - 1;
      a_src[p] = g.A + (int64_t)row * g.pitch + lseg;
    }
#pragma unroll
    for (int p = 0; p < PB; ++p) {
      int row = n0 + lr + RPP * p;
      row = row < g.N ? row : g.N - 1;
      b_src[p] = g.B + (int64_t)row * g.pitch + lseg;
    }
  };
  // Row factors of the current tile; visible to every wave after the next barrier.
  auto fill_rowfac = [&]() {
    if (g.out_f32) {
      // INT4 accumulators carry an exact factor 256 (a power of two: folding it into the
      // row factor gives the same fp32 result as shifting the integer first)
      const float cs = (*g.col_scale) * g.inv_n * (INT4 ? 1.0f / 256.0f : 1.0f);
      for (int i = tid; i < BM; i += NT)
        s_rowfac[i] = m0 + i < g.M ? g.row_scale[(int64_t)(m0 + i) * g.row_stride] * cs : 0.0f;
    }
  };
  v4i ra[PA], rb[PB];
  auto load_stage = [&](int kt) {
    const int64_t off = (int64_t)kt * BKB;
#pragma unroll
    for (int p = 0; p < PA; ++p) ra[p] = *reinterpret_cast<const v4i*>(a_src[p] + off);
#pragma unroll
    for (int p = 0; p < PB; ++p) rb[p] = *reinterpret_cast<const v4i*>(b_src[p] + off);
  };
  auto store_stage = [&](int buf) {
#pragma unroll
    for (int p = 0; p < PA; ++p)
      *reinterpret_cast<v4i*>(&As[buf * BM * LP + RPP * p * LP + st_off]) = ra[p];
#pragma unroll
    for (int p = 0; p < PB; ++p)
      *reinterpret_cast<v4i*>(&Bs[buf * BN * LP + RPP * p * LP + st_off]) = rb[p];
  };

  acc_t acc[TM][TN];
  auto zero_acc = [&]() {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;
  };

  int a_off[KS], b_off[KS];  // fragment of K slice ks: chunk 2*ks + lane/32 of row lane%32
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    const int pos = 16 * ((2 * ks + (lane >> 5)) ^ swz(lane & 31));
    a_off[ks] = (wm0 + (lane & 31)) * LP + pos;
    b_off[ks] = (wn0 + (lane & 31)) * LP + pos;
  }
  v4i fa[TM], fb[TN];  // raw 16-byte fragments in flight (INT4 only)
  // One K slice = NM matrix instructions; everything else the slice has to issue is
  // cut into "events" that are emitted, in a fixed order, between those instructions:
  //   slice 0 of a stage: NG x (LDS store of stage it+1, global load of stage it+2),
  //   every slice: NR LDS fragment reads of the next slice, then (INT4) 2*NR widenings
  //   of half a fragment each.  sched_barrier(0) after every step pins the order.
  constexpr int NM = TM * TN * (INT4 ? 2 : 1);
  constexpr int NR = TM + TN;
  constexpr int NG = PA + PB;
  constexpr int NW = INT4 ? 2 * NR : 0;

  Operands<TM, TN, INT4> u0, u1;
  // event bodies; every index is a compile-time constant so all arrays stay in registers
  auto read_one = [&](Operands<TM, TN, INT4>& un, int buf, int ks, auto fc) {
    constexpr int f = decltype(fc)::value;
    v4i val;
    if constexpr (f < TM) val = *reinterpret_cast<const v4i*>(&As[buf * BM * LP + a_off[ks] + f * 32 * LP]);
    else val = *reinterpret_cast<const v4i*>(&Bs[buf * BN * LP + b_off[ks] + (f - TM) * 32 * LP]);
    if constexpr (INT4) {
      if constexpr (f < TM) fa[f] = val; else fb[f - TM] = val;
    } else {
      if constexpr (f < TM) un.a[0][f] = val; else un.b[0][f - TM] = val;
    }
  };
  auto widen_half = [&](Operands<TM, TN, INT4>& un, auto ec) {  // two dwords of fragment e/2
    if constexpr (INT4) {
      constexpr int e = decltype(ec)::value;
      constexpr int f = e >> 1, d0 = (e & 1) * 2;
      static_for<2>([&](auto dc) {
        constexpr int d = d0 + decltype(dc)::value;
        if constexpr (f < TM) {
          const unsigned x = (unsigned)fa[f][d];
          un.a[0][f][d] = (int)((x << 4) & 0xF0F0F0F0u);
          un.a[1][f][d] = (int)(x & 0xF0F0F0F0u);
        } else {
          const unsigned x = (unsigned)fb[f - TM][d];
          un.b[0][f - TM][d] = (int)((x << 4) & 0xF0F0F0F0u);
          un.b[1][f - TM][d] = (int)(x & 0xF0F0F0F0u);
        }
      });
    }
  };
  auto store_one = [&](int buf, auto pc) {
    constexpr int p = decltype(pc)::value;
    if constexpr (p < PA) *reinterpret_cast<v4i*>(&As[buf * BM * LP + RPP * p * LP + st_off]) = ra[p];
    else *reinterpret_cast<v4i*>(&Bs[buf * BN * LP + RPP * (p - PA) * LP + st_off]) = rb[p - PA];
  };
  auto load_one = [&](int64_t off, auto pc) {
    constexpr int p = decltype(pc)::value;
    if constexpr (p < PA) ra[p] = *reinterpret_cast<const v4i*>(a_src[p] + off);
    else rb[p - PA] = *reinterpret_cast<const v4i*>(b_src[p - PA] + off);
  };
  // one K slice: matrix instructions on `uc`, events that prepare `un`
  auto slice = [&](auto ksc, Operands<TM, TN, INT4>& uc, Operands<TM, TN, INT4>& un, int cur,
                   int nxt, int64_t off2) {
    constexpr int ks = decltype(ksc)::value;
    constexpr bool last = ks + 1 == KS;
    constexpr int NS = ks == 0 ? 2 * NG : 0;   // store/load events come first
    constexpr int NE = NS + NR + NW;
    if constexpr (last) __syncthreads();  // everyone has written `nxt` and finished reading `cur`
    __builtin_amdgcn_sched_barrier(0);
    static_for<NM>([&](auto qc) {
      constexpr int q = decltype(qc)::value;
      constexpr int E0 = (q * NE + NM - 1) / NM;           // events e with e*NM < (q+1)*NE ...
      constexpr int E1 = ((q + 1) * NE + NM - 1) / NM;     // ... not yet emitted
      static_for<E1 - E0>([&](auto dc) {
        constexpr int e = E0 + decltype(dc)::value;
        if constexpr (e < NS) {
          if constexpr ((e & 1) == 0) store_one(nxt, std::integral_constant<int, e / 2>{});
          else load_one(off2, std::integral_constant<int, e / 2>{});
        } else if constexpr (e < NS + NR) {
          read_one(un, last ? nxt : cur, last ? 0 : ks + 1, std::integral_constant<int, e - NS>{});
        } else {
          widen_half(un, std::integral_constant<int, e - NS - NR>{});
        }
      });
      constexpr int h = q / (TM * TN), i = (q % (TM * TN)) / TN, j = q % TN;
      if constexpr (BF16)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, uc.a[h][i]),
                                                            __builtin_bit_cast(v8bf, uc.b[h][j]),
                                                            acc[i][j], 0, 0, 0);
      else
        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(uc.a[h][i], uc.b[h][j], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    });
  };
  // acc += K stages [k_begin, k_end) of the current tile.  The caller has put a barrier
  // between the last use of LDS and this call.
  auto main_loop = [&](int k_begin, int k_end) {
    const int nk = k_end - k_begin;
    if (nk <= 0) return;
    load_stage(k_begin);
    store_stage(0);
    load_stage(k_begin + (nk > 1 ? 1 : 0));
    __syncthreads();
    static_for<NR>([&](auto fc) { read_one(u0, 0, 0, fc); });
    static_for<(NW > 0 ? NW : 1)>([&](auto ec) { widen_half(u0, ec); });
    for (int it = 0; it < nk; ++it) {
      const int cur = it & 1, nxt = cur ^ 1;
      int kt2 = k_begin + it + 2;
      kt2 = kt2 < k_end ? kt2 : k_end - 1;  // tail iterations re-load a valid stage (unused)
      const int64_t off2 = (int64_t)kt2 * BKB;
      static_for<KS>([&](auto ksc) {
        constexpr int ks = decltype(ksc)::value;
        if constexpr ((ks & 1) == 0) slice(ksc, u0, u1, cur, nxt, off2);
        else slice(ksc, u1, u0, cur, nxt, off2);
      });
    }
  };

  // Epilogue.  Accumulator register v of a 32x32 tile: row 8*(v/4) + 4*(lane/32) + v%4,
  // column lane%32, so each register is stored as 32-float (128-byte) row segments.
  // The row factors come from LDS (filled before the main loop): a global load per row
  // here could not be hoisted above the output stores and would serialise on L2 latency.
  // Offsets within the tile are 32-bit on top of a uniform base pointer.
  auto epilogue = [&]() {
    // Split-K runs this after loops: an opaque copy of the lane index keeps the compiler
    // from hoisting the ~100 output addresses out of them (they would be live, in
    // registers, across the main loop).
    int ln = lane;
    if constexpr (SPLITK) asm volatile("" : "+v"(ln));
    const int lane = ln;
    const int nl0 = wn0 + (lane & 31);
    if (g.out_f32 && m0 + BM <= g.M && n0 + BN <= g.N) {
      // A tile that lies inside the output (all but the last tile row and column): no bound
      // checks, and one address per lane for the whole tile: the row within the tile is a
      // uniform offset on the base pointer, the column block a constant.  The checked form
      // below costs a dozen instructions and two branches per element, 13 us per 256x256
      // tile where this one takes 3.
      const unsigned lane_byte = 4u * (unsigned)((wm0 + 4 * (lane >> 5)) * g.N + nl0);   // < 2^32: inside one tile
      char* const tile = reinterpret_cast<char*>(g.out_f32 + ((int64_t)m0 * g.N + n0));
      auto store_tile = [&](auto nt_c) {
        constexpr bool NT = decltype(nt_c)::value;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            typedef float v4f __attribute__((ext_vector_type(4)));
            const v4f rs4 = *reinterpret_cast<const v4f*>(&s_rowfac[wm0 + i * 32 + 8 * q + 4 * (lane >> 5)]);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              char* const row = tile + (int64_t)(i * 32 + 8 * q + r) * g.N * 4;   // uniform
              if constexpr (NT) {
                // written as an instruction: two branches that differ only in a store's cache
                // hint are merged by the compiler, and the hint is lost
                float* dst = reinterpret_cast<float*>(row + lane_byte);
                static_for<TN>([&](auto jc) {
                  constexpr int j = decltype(jc)::value;
                  float val;
                  if constexpr (BF16) val = acc[i][j][4 * q + r] * rs4[r];
                  else val = (float)acc[i][j][4 * q + r] * rs4[r];
                  store_streaming<j * 128>(dst, val);
                });
              } else {
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                  float* const dst = reinterpret_cast<float*>(row + j * 128 + lane_byte);
                  if constexpr (BF16) *dst = acc[i][j][4 * q + r] * rs4[r];
                  else *dst = (float)acc[i][j][4 * q + r] * rs4[r];
                }
              }
            }
          }
        }
      };
      // Streaming stores keep the output out of the way of the operand tiles in L2 (with a
      // short K the 4 MB of an XCD otherwise lose the weight operand to the output between two
      // bands of tiles); with a long K per tile they measured slower than plain stores.
      if (g.stream_out) store_tile(std::true_type{});
      else store_tile(std::false_type{});
    } else if (g.out_f32) {
      float* obase = g.out_f32 + ((int64_t)m0 * g.N + n0);
#pragma unroll
      for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int ml = wm0 + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
          if (m0 + ml >= g.M) continue;
          const float rs = s_rowfac[ml];
          const int row_off = ml * g.N + nl0;
#pragma unroll
          for (int j = 0; j < TN; ++j)
            if (n0 + nl0 + j * 32 < g.N) obase[row_off + j * 32] = (float)acc[i][j][v] * rs;
        }
      }
    } else {
      int32_t* obase = g.out_i32 + ((int64_t)m0 * g.N + n0);
#pragma unroll
      for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int ml = wm0 + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
          if (m0 + ml >= g.M) continue;
          const int row_off = ml * g.N + nl0;
#pragma unroll
          for (int j = 0; j < TN; ++j)
            if (n0 + nl0 + j * 32 < g.N) {
              if constexpr (BF16) obase[row_off + j * 32] = __float_as_int(acc[i][j][v]);
              else obase[row_off + j * 32] = INT4 ? (acc[i][j][v] >> 8) : acc[i][j][v];
            }
        }
      }
    }
  };

  if constexpr (!SPLITK) {
    int tm, tn;
    tile_of_position(g, xcd_contiguous(blockIdx.x, g.tiles_m * g.tiles_n), tm, tn);
    set_tile(tm, tn);
    fill_rowfac();
    zero_acc();
    main_loop(0, g.nk_total);   // has a barrier when there is any stage; else acc = 0 ...
    if (g.nk_total <= 0) __syncthreads();   // ... and the row factors still need one
    epilogue();
  } else {
    constexpr int IMG = BM * BN;
    const int tiles = g.tiles_m * g.tiles_n, nk = g.nk_total, S = g.split;
    int z = blockIdx.x / tiles;   // slices in dispatch order: owners (z = S - 1) start last
    int tm, tn, t;
    if (g.xcd_cols < 0) {
      // S divides 8: the XCDs are dealt to the slices, 8 / S to each, and the XCDs of a slice
      // share its tiles by row bands.  An A row band of a slice is then fetched by one XCD, a B
      // band by 8 / S of them: the whole GEMM fetches A once and B 8 / S times.
      const int per = 8 / S, x = blockIdx.x & 7, j = blockIdx.x >> 3;   // XCD, index within it
      z = x / per;
      t = (x % per) * (tiles / per) + j;
      tm = t / g.tiles_n;
      tn = t % g.tiles_n;
    } else if (g.xcd_cols > 0) {
      // Workgroups go to the eight XCDs in turn, each with an L2 of its own.  Every XCD gets one
      // rectangle of the tile grid, in every slice the same one: an operand row band is then
      // fetched by the xcd_cols XCDs that share it and by no other (with the band walk below the
      // bands of a small grid end up on three to eight of them).
      t = blockIdx.x - z * tiles;          // tiles is a multiple of 8 here: XCD = t % 8
      const int x = t & 7, j = t >> 3;
      const int rm = g.tiles_m / (8 / g.xcd_cols), rn = g.tiles_n / g.xcd_cols;
      tm = (x / g.xcd_cols) * rm + j % rm;
      tn = (x % g.xcd_cols) * rn + j / rm;
    } else {
      t = xcd_contiguous(blockIdx.x - z * tiles, tiles);
      tile_of_position(g, t, tm, tn);
    }
    auto slice_begin = [&](int zz) { return (int)(((int64_t)zz * nk) / S); };
    const bool owned = z == S - 1;
    set_tile(tm, tn);
    if (owned) fill_rowfac();
    zero_acc();
    // own slice first, then the earlier ones: taken from their workgroups' images, or, when
    // one does not show up in time, computed here
    int zz = z;
    while (true) {
      main_loop(slice_begin(zz), slice_begin(zz + 1));
      bool more = false;
      while (owned && zz > 0) {
        --zz;
        const int slot = t * (S - 1) + zz;
        if (tid == 0) {
          const unsigned long long want = effective_tag(g.tag, g.epoch);
          const long long start = wall_clock64();
          bool seen;
          do {
            seen = __hip_atomic_load(&g.flags[slot], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == want;
          } while (!seen && wall_clock64() - start < g.wait_ticks);
          s_seen = seen;
        }
        __syncthreads();
        const bool seen = s_seen != 0;
        __syncthreads();   // everyone has read s_seen before it can be rewritten
        if (!seen) { more = true; break; }
        // up to four 32x32 tiles' worth of loads in flight at a time (one memory round trip
        // for the 128x128 tile; more would not fit next to the larger tiles' accumulators)
        int t_img = tid;
        asm volatile("" : "+v"(t_img));   // addresses are computed here, not before the loop
        const int32_t* img = g.partial + (int64_t)slot * IMG + t_img;
        constexpr int QG = TM * TN < 4 ? TM * TN : 4;
        static_assert(TM * TN % QG == 0, "groups of accumulator tiles");
        static_for<TM * TN / QG>([&](auto gc) {
          constexpr int q0 = decltype(gc)::value * QG;
          int part[QG][16];
#pragma unroll
          for (int q = 0; q < QG; ++q)
#pragma unroll
            for (int v = 0; v < 16; ++v)
              part[q][v] = __hip_atomic_load(&img[((q0 + q) * 16 + v) * NT], __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
          for (int q = 0; q < QG; ++q)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[(q0 + q) / TN][(q0 + q) % TN][v] += part[q][v];
          __builtin_amdgcn_sched_barrier(0);
        });
      }
      if (!more) break;
      __syncthreads();   // LDS of the last main loop is free again
    }
    if (owned) {
      if (nk < S) __syncthreads();   // no slice had a stage (and so no barrier) of its own
      epilogue();
    } else {
      const int slot = t * (S - 1) + z;
      int t_img = tid;
      asm volatile("" : "+v"(t_img));
      int32_t* mine = g.partial + (int64_t)slot * IMG + t_img;
      static_for<TM * TN>([&](auto qc) {
        constexpr int q = decltype(qc)::value;
#pragma unroll
        for (int v = 0; v < 16; ++v)
          __hip_atomic_store(&mine[(q * 16 + v) * NT], acc[q / TN][q % TN][v], __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
        __builtin_amdgcn_sched_barrier(0);
      });
      // Image and flag travel as device-scope accesses that bypass the per-XCD L2, so no
      // cache-wide write-back or invalidate (which would also evict every workgroup's
      // operand tiles) is needed: the flag is stored once every thread's image stores have
      // been acknowledged.
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
      if (tid == 0)
        __hip_atomic_store(&g.flags[slot], effective_tag(g.tag, g.epoch), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

}  // namespace hot
