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
// is ever transposed in a separate pass.  HBM-bound.  The tensor-wide scale is a true
// dependency on every element: tensors whose kept values fit the register files of the
// resident workgroups are read once (col_quant_onepass_kernel: the maxima are exchanged
// through memory while the values wait in registers); larger ones are read twice (abs-max
// pass leaving one partial maximum per workgroup, quantise pass reducing them itself).
// Neither form needs atomics on data or zero-initialised memory.
#pragma once
#include <type_traits>

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

// Natural-order index of the row of H_n with j sign changes: bit-reversed Gray code.
__host__ __device__ constexpr int lowpass_row(int n, int j) {
  const int g = j ^ (j >> 1);
  int r = 0;
  for (int b = 1, t = n >> 1; b < n; b <<= 1, t >>= 1)
    if (g & b) r |= t;
  return r;
}

// First row of block gb and how many of its N rows are real tokens (the rest are zeros).
template <int N>
__device__ __forceinline__ void block_rows(const RowTiling& t, int64_t gb, int64_t& first, int& valid) {
  if (t.S == 0) {
    first = gb * N;
    valid = N;
  } else {
    const int64_t b = gb / t.bps;
    const int64_t j = gb - b * t.bps;
    first = b * t.S + j * N;
    const int64_t left = t.S - j * N;
    valid = left < N ? (int)left : N;
  }
}

// Which kept-row list the kernel was compiled for.
enum KeepKind {
  kKeepGeneric = 0,   // any list, from the KeepMap argument; INT8 codes, one LDS byte each
  kKeepLowHalf = 1,   // the n/2 rows of lowest sequency, in sequency order; INT8
  kKeepAll8 = 2,      // all rows, natural order; INT8
  kKeepAll4 = 3,      // all rows, natural order; INT4, two codes per byte
};

// Load one block (N rows x VEC columns per lane) and transform it in registers.
// N rows starting at `src` (row stride C floats), `col` floats into each row.  Rows
// k >= valid are the zero padding of a sample's last block: they re-read the last real row
// (never past it) and are zeroed.  The full block keeps compile-time row offsets; the
// padded one steps a pointer, so neither pays a 64-bit multiply per row.
template <int N, class VT>
__device__ __forceinline__ void load_n_rows(const float* __restrict__ src, int64_t C, uint32_t col,
                                            int valid, VT (&q)[N]) {
  if (valid >= N) {
#pragma unroll
    for (int k = 0; k < N; ++k) q[k] = *reinterpret_cast<const VT*>(src + (int64_t)k * C + col);
  } else {
    const float* p = src;
#pragma unroll
    for (int k = 0; k < N; ++k) {
      q[k] = *reinterpret_cast<const VT*>(p + col);
      if (k >= valid) q[k] = VT{};
      if (k + 1 < valid) p += C;
    }
  }
}

template <int N, int VEC>
__device__ __forceinline__ void load_block_fwht(const float* __restrict__ src, int64_t C, int valid,
                                                float (&v)[VEC][N]) {
  using VT = typename VecT<VEC>::type;
  VT q[N];
  load_n_rows<N, VT>(src, C, 0u, valid, q);
#pragma unroll
  for (int k = 0; k < N; ++k) {
    float o[VEC];
    unpack_vec<VEC>(q[k], o);
#pragma unroll
    for (int vi = 0; vi < VEC; ++vi) v[vi][k] = o[vi];
  }
#pragma unroll
  for (int vi = 0; vi < VEC; ++vi) fwht_regs<N>(v[vi]);
}

// Quantise the block a lane holds (v[vi][k]: column vi of the lane, transformed row k)
// and drop the kept rows' codes into the LDS tile at byte `off` of the lane's rows.
template <int N, int VEC, int KIND>
__device__ __forceinline__ void store_block_codes(const float (&v)[VEC][N], uint8_t* tile, int lane,
                                                  int off, int TBP, const KeepMap& map, float inv,
                                                  int rounding) {
  constexpr int BITS = KIND == kKeepAll4 ? 4 : 8;
  constexpr int QMAX = (1 << (BITS - 1)) - 1;
#pragma unroll
  for (int vi = 0; vi < VEC; ++vi) {
    uint8_t* dst = tile + (vi * 64 + lane) * TBP + off;
    if constexpr (KIND == kKeepGeneric) {
#pragma unroll
      for (int k = 0; k < N; ++k) {
        const int p = map.pos[k];
        if (p >= 0) dst[p] = (uint8_t)quant_code(v[vi][k], inv, QMAX, rounding);
      }
    } else if constexpr (KIND == kKeepAll4) {
#pragma unroll
      for (int k8 = 0; k8 < N / 8; ++k8) {
        int c[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) c[e] = quant_code(v[vi][k8 * 8 + e], inv, QMAX, rounding);
        reinterpret_cast<uint32_t*>(dst)[k8] = pack8_codes4(c);
      }
    } else {
      constexpr int RK = KIND == kKeepLowHalf ? N / 2 : N;
#pragma unroll
      for (int j4 = 0; j4 < RK / 4; ++j4) {
        int c[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int j = j4 * 4 + e;
          const int k = KIND == kKeepLowHalf ? lowpass_row(N, j) : j;
          c[e] = quant_code(v[vi][k], inv, QMAX, rounding);
        }
        reinterpret_cast<uint32_t*>(dst)[j4] = pack4_codes8(c[0], c[1], c[2], c[3]);
      }
    }
  }
}

// Write the LDS tile out as contiguous runs per column; the last row tile also
// zero-fills up to the pitch.
template <int VEC>
__device__ __forceinline__ void write_out_tile(const uint8_t* tile, int TB, int TBP, int64_t tx,
                                               int64_t ty, int64_t nblk, int kbw, int64_t C,
                                               int64_t pitch, uint8_t* __restrict__ codes) {
  constexpr int CT = 64 * VEC;
  const int tid = threadIdx.x;
  const int64_t tile_off = ty * TB;
  int64_t cover = (ty == (nblk + 4 * kbw - 1) / (4 * kbw) - 1) ? pitch - tile_off : TB;
  if (cover > pitch - tile_off) cover = pitch - tile_off;
  const int cdw = (int)(cover >> 2), tdw = TB >> 2;
  for (int idx = tid; idx < CT * cdw; idx += 256) {
    const int col = idx / cdw, dw = idx - col * cdw;
    const int64_t c = tx * CT + col;
    if (c < C) {
      const int row = (col % VEC) * 64 + col / VEC;
      const uint32_t val = dw < tdw ? *reinterpret_cast<const uint32_t*>(tile + row * TBP + 4 * dw) : 0u;
      *reinterpret_cast<uint32_t*>(codes + c * pitch + tile_off + 4 * dw) = val;
    }
  }
}

// Largest kept |value| of a transformed block.
template <int N, int VEC, int KIND>
__device__ __forceinline__ float kept_absmax(const float (&v)[VEC][N], const KeepMap& map) {
  float m = 0.0f;
#pragma unroll
  for (int k = 0; k < N; ++k) {
    bool kept;
    if constexpr (KIND == kKeepGeneric) kept = map.pos[k] >= 0;
    else if constexpr (KIND == kKeepLowHalf) kept = (k & 1) == 0;  // even natural rows
    else kept = true;
    if (kept) {
#pragma unroll
      for (int vi = 0; vi < VEC; ++vi) m = fmaxf(m, fabsf(v[vi][k]));
    }
  }
  return m;
}

// Column transform restricted to the even natural rows (the N/2 lowest sequencies):
// those outputs only take the sum branch of stage h = 1, so s[j] = v[2j] + v[2j+1]
// followed by the N/2-point transform gives output row 2j' at s[j'] with the same
// additions in the same order as the full transform.
template <int N>
__device__ __forceinline__ void fwht_even_rows(const float (&v)[N], float (&s)[N / 2]) {
#pragma unroll
  for (int j = 0; j < N / 2; ++j) s[j] = v[2 * j] + v[2 * j + 1];
  fwht_regs<N / 2>(s);
}

// Values a lane keeps per column of a block: only the kept half when that is known at
// compile time.
template <int N, int KIND>
constexpr int kept_vals() { return KIND == kKeepLowHalf ? N / 2 : N; }

// The N rows of one block as loaded (zeros when `ok` is false; nothing is dereferenced
// then).  `rows` is wave-uniform (the block's first row at the tile's first column), `col`
// the lane's 32-bit column offset, so the row stride is added on the scalar unit.
template <int N, int VEC>
__device__ __forceinline__ void load_rows(const float* __restrict__ rows, int64_t C, uint32_t col,
                                          bool ok, int valid, typename VecT<VEC>::type (&q)[N]) {
  using VT = typename VecT<VEC>::type;
  if (ok) {
    load_n_rows<N, VT>(rows, C, col, valid, q);
  } else {
#pragma unroll
    for (int k = 0; k < N; ++k) q[k] = VT{};
  }
}

// Transform loaded rows into kept form (see load_block_kept).
template <int N, int VEC, int KIND>
__device__ __forceinline__ void transform_kept(const typename VecT<VEC>::type (&q)[N],
                                               float (&v)[VEC][kept_vals<N, KIND>()]) {
  if constexpr (KIND == kKeepLowHalf) {
#pragma unroll
    for (int j = 0; j < N / 2; ++j) {
      float a[VEC], b[VEC];
      unpack_vec<VEC>(q[2 * j], a);
      unpack_vec<VEC>(q[2 * j + 1], b);
#pragma unroll
      for (int vi = 0; vi < VEC; ++vi) v[vi][j] = a[vi] + b[vi];
    }
#pragma unroll
    for (int vi = 0; vi < VEC; ++vi) fwht_regs<N / 2>(v[vi]);
  } else {
#pragma unroll
    for (int k = 0; k < N; ++k) {
      float o[VEC];
      unpack_vec<VEC>(q[k], o);
#pragma unroll
      for (int vi = 0; vi < VEC; ++vi) v[vi][k] = o[vi];
    }
#pragma unroll
    for (int vi = 0; vi < VEC; ++vi) fwht_regs<N>(v[vi]);
  }
}

// Load one block and return its transformed values in kept form: all N natural rows, or
// (kKeepLowHalf) the even natural rows, row 2j' at index j'.
template <int N, int VEC, int KIND>
__device__ __forceinline__ void load_block_kept(const float* __restrict__ src, int64_t C, int valid,
                                                float (&v)[VEC][kept_vals<N, KIND>()]) {
  if constexpr (KIND == kKeepLowHalf) {
    float full[VEC][N];
    using VT = typename VecT<VEC>::type;
    VT q[N];
    load_n_rows<N, VT>(src, C, 0u, valid, q);
#pragma unroll
    for (int k = 0; k < N; ++k) {
      float o[VEC];
      unpack_vec<VEC>(q[k], o);
#pragma unroll
      for (int vi = 0; vi < VEC; ++vi) full[vi][k] = o[vi];
    }
#pragma unroll
    for (int vi = 0; vi < VEC; ++vi) fwht_even_rows<N>(full[vi], v[vi]);
  } else {
    load_block_fwht<N, VEC>(src, C, valid, v);
  }
}

template <int N, int VEC, int KIND>
__device__ __forceinline__ float kept_form_absmax(const float (&v)[VEC][kept_vals<N, KIND>()],
                                                  const KeepMap& map) {
  if constexpr (KIND == kKeepLowHalf) {
    float m = 0.0f;
#pragma unroll
    for (int k = 0; k < N / 2; ++k) {
#pragma unroll
      for (int vi = 0; vi < VEC; ++vi) m = fmaxf(m, fabsf(v[vi][k]));
    }
    return m;
  } else {
    return kept_absmax<N, VEC, KIND>(v, map);
  }
}

template <int N, int VEC, int KIND>
__device__ __forceinline__ void store_kept_form_codes(const float (&v)[VEC][kept_vals<N, KIND>()],
                                                      uint8_t* tile, int lane, int off, int TBP,
                                                      const KeepMap& map, float inv, int rounding) {
  if constexpr (KIND == kKeepLowHalf) {
#pragma unroll
    for (int vi = 0; vi < VEC; ++vi) {
      uint32_t* dst = reinterpret_cast<uint32_t*>(tile + (vi * 64 + lane) * TBP + off);
#pragma unroll
      for (int j4 = 0; j4 < N / 8; ++j4) {
        int c[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) c[e] = quant_code(v[vi][lowpass_row(N, j4 * 4 + e) >> 1], inv, 127, rounding);
        dst[j4] = pack4_codes8(c[0], c[1], c[2], c[3]);
      }
    }
  } else {
    store_block_codes<N, VEC, KIND>(v, tile, lane, off, TBP, map, inv, rounding);
  }
}

// Maximum over the 256 threads of a workgroup, returned to all of them.
__device__ __forceinline__ float workgroup_max(float m) {
  __shared__ float s_wg[4];
  m = wave_max(m);
  if ((threadIdx.x & 63) == 0) s_wg[threadIdx.x >> 6] = m;
  __syncthreads();
  m = fmaxf(fmaxf(s_wg[0], s_wg[1]), fmaxf(s_wg[2], s_wg[3]));
  __syncthreads();
  return m;
}

// Abs-max pass.  Tiles of (4*kbw blocks) x (64*VEC columns) are dealt to a capped
// grid; partials[blockIdx.x] = the workgroup's maximum over its tiles.
// Abs-max pass.  The four waves of a workgroup take adjacent column stripes of the same
// blocks, so a row of the workgroup's tile is 4 * 64 * VEC consecutive floats requested at
// about the same time (longer runs per DRAM page than four waves on four different row
// blocks: 6.0 against 5.3 TB/s on a 721 MB tensor when the kernel runs alone, 152 against
// 157 us between the GEMMs of a training step); a wave goes through `kbw` consecutive
// blocks, workgroups loop over the tiles.
template <int N, int VEC, int KIND>
__global__ __launch_bounds__(256) void col_absmax_kernel(const float* __restrict__ x, RowTiling rt,
                                                         int64_t C, KeepMap map, int kbw,
                                                         float* __restrict__ partials) {
  constexpr int CT = 64 * VEC;
  __shared__ float s_max[4];
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int64_t nblk = rt.nblk;
  const int64_t tiles_x = (C + 4 * CT - 1) / (4 * CT);
  const int64_t tiles_y = (nblk + kbw - 1) / kbw;
  float m = 0.0f;
  for (int64_t t = blockIdx.x; t < tiles_x * tiles_y; t += gridDim.x) {
    const int64_t tx = t % tiles_x, ty = t / tiles_x;
    const int64_t c0 = tx * 4 * CT + w * CT + lane * VEC;
    if (c0 >= C) continue;
    for (int kb = 0; kb < kbw; ++kb) {
      const int64_t gb = ty * kbw + kb;
      if (gb >= nblk) break;
      float v[VEC][kept_vals<N, KIND>()];
      int64_t first;
      int valid;
      block_rows<N>(rt, gb, first, valid);
      load_block_kept<N, VEC, KIND>(x + first * C + c0, C, valid, v);
      m = fmaxf(m, kept_form_absmax<N, VEC, KIND>(v, map));
    }
  }
  m = wave_max(m);
  if (lane == 0) s_max[w] = m;
  __syncthreads();
  if (tid == 0) partials[blockIdx.x] = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));
}

// Quantise pass: one tile per workgroup.  LDS tile: row (vi*64 + lane) holds the code
// bytes of column lane*VEC + vi (odd dword pitch: conflict-free for both the strided
// writes and the row-wise read-out).
template <int N, int VEC, int KIND>
__global__ __launch_bounds__(256) void col_quant_kernel(
    const float* __restrict__ x, RowTiling rt, int64_t C, KeepMap map, int r, int rounding, int kbw,
    const float* __restrict__ partials, int npartials, uint8_t* __restrict__ codes, int64_t pitch,
    float* __restrict__ scale) {
  constexpr int CT = 64 * VEC;
  constexpr int BITS = KIND == kKeepAll4 ? 4 : 8;
  constexpr int QMAX = (1 << (BITS - 1)) - 1;
  extern __shared__ __align__(16) uint8_t tile[];
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int bpb = KIND == kKeepGeneric ? r : (KIND == kKeepLowHalf ? N / 2 : (KIND == kKeepAll8 ? N : N / 2));
  const int TB = 4 * kbw * bpb;      // code bytes per column in this tile
  const int TBP = TB + 4;            // odd number of dwords
  const int64_t nblk = rt.nblk;
  const int64_t tiles_x = (C + CT - 1) / CT;
  // Last tile first: the abs-max pass ended on the rows with the highest index, and what it read
  // last is what the 256 MB memory-side cache still holds.
  const int64_t bid = (int64_t)gridDim.x - 1 - blockIdx.x;
  const int64_t tx = bid % tiles_x, ty = bid / tiles_x;
  const int64_t c0 = tx * CT + lane * VEC;
  const bool col_ok = c0 < C;

  const float amax = block_max_of(partials, npartials);
  const float inv = quant_inv(amax, QMAX);
  if (blockIdx.x == 0 && tid == 0) *scale = quant_scale(amax, QMAX);
  // slots of blocks past the end must read back as zero codes
  if ((ty + 1) * 4 * kbw > nblk) {
    for (int i = tid; i < CT * TBP / 4; i += 256) reinterpret_cast<uint32_t*>(tile)[i] = 0u;
    __syncthreads();
  }

  for (int kb = 0; kb < kbw; ++kb) {
    const int slot = w * kbw + kb;
    const int64_t gb = ty * 4 * kbw + slot;
    if (gb >= nblk || !col_ok) continue;
    float v[VEC][kept_vals<N, KIND>()];
    int64_t first;
    int valid;
    block_rows<N>(rt, gb, first, valid);
    load_block_kept<N, VEC, KIND>(x + first * C + c0, C, valid, v);
    store_kept_form_codes<N, VEC, KIND>(v, tile, lane, slot * bpb, TBP, map, inv, rounding);
  }
  __syncthreads();

  write_out_tile<VEC>(tile, TB, TBP, tx, ty, nblk, kbw, C, pitch, codes);
}

// Single-pass variant for tensors that fit in the register files of the resident
// workgroups: every workgroup keeps its transformed tile (4*KB blocks x 64*VEC columns)
// in registers, publishes the tile's kept abs-max, collects everybody else's, and
// quantises from registers: one read of the input, one launch.
//
// Exchange: workgroup b owns two 64-bit words, (upper half of the launch tag << 32 | float
// bits) and (lower half << 32 | the same float bits), each written with one device-scope
// atomic store.  A reader takes the value once both words carry this launch's halves and
// the same value, so the memory needs no initialisation, the two words need no ordering
// between them, and a leftover of any earlier launch would have to match all 64 tag bits.  Waiting is bounded: after `wait_ticks` of the 100 MHz
// wall clock a workgroup computes the maxima still missing itself (each is a pure
// function of that tile's input), so every wave finishes whether or not the other
// workgroups are resident, and the result does not depend on who computed what.
// Code bytes per block and column when the kept list is known at compile time.
template <int N, int KIND>
constexpr int static_bpb() { return KIND == kKeepAll8 ? N : N / 2; }

// The codes of one column of a block (kept form) packed in output order.
template <int N, int KIND, int ROUNDING>
__device__ __forceinline__ void pack_kept_codes(const float (&v)[kept_vals<N, KIND>()], float inv,
                                                uint32_t (&out)[static_bpb<N, KIND>() / 4]) {
  static_assert(KIND != kKeepGeneric, "compile-time kept lists only");
  if constexpr (KIND == kKeepAll4) {
#pragma unroll
    for (int k8 = 0; k8 < N / 8; ++k8) {
      int c[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) c[e] = quant_code(v[k8 * 8 + e], inv, 7, ROUNDING);
      out[k8] = pack8_codes4(c);
    }
  } else {
#pragma unroll
    for (int j4 = 0; j4 < static_bpb<N, KIND>() / 4; ++j4) {
      int c[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int j = j4 * 4 + e;
        c[e] = quant_code(v[KIND == kKeepLowHalf ? (lowpass_row(N, j) >> 1) : j], inv, 127, ROUNDING);
      }
      out[j4] = pack4_codes8(c[0], c[1], c[2], c[3]);
    }
  }
}

// Register plan of the single-pass kernel: two waves share a SIMD (256 registers each);
// a lane keeps KB * VEC * kept values for the whole kernel plus DEPTH row buffers of one
// block (the next block's loads in flight under the current block's butterflies when that
// still fits).
// Whether the 4 * KB blocks of a workgroup give every output row a whole number of
// 128-byte lines (the rows' pitch is a multiple of 128 bytes).
template <int N, int KIND, int KB>
constexpr bool onepass_whole_lines() {
  if constexpr (KIND == kKeepGeneric) return false;
  else return (4 * KB * static_bpb<N, KIND>()) % 128 == 0;
}

template <int N, int VEC, int KIND, int KB>
constexpr int onepass_kept_regs() { return KB * VEC * kept_vals<N, KIND>(); }
template <int N, int VEC, int KIND, int KB>
constexpr int onepass_depth() { return (KB > 1 && onepass_kept_regs<N, VEC, KIND, KB>() + 2 * N * VEC <= 224) ? 2 : 1; }
constexpr int kOnepassMaxKept = 160;

// Bytes of dynamic LDS: the code tile, or (before the tile is filled) one column of
// per-lane staging for the recomputation of another workgroup's maximum, used by one wave
// at a time (that path is rare; a small footprint keeps more workgroups per compute unit).
template <int N, int VEC, int KIND>
constexpr size_t onepass_stage_bytes() { return (size_t)kept_vals<N, KIND>() * 64 * VEC * 4; }

// Whether a lane of the single-pass kernel stores its codes straight from registers: the
// kept list is known at compile time and the lane's KB blocks give at least 48 consecutive
// output bytes (shorter runs are cheaper to gather through the LDS tile).
template <int N, int KIND, int KB>
constexpr bool onepass_direct_store() {
  if constexpr (KIND == kKeepGeneric) return false;
  else return static_bpb<N, KIND>() % 8 == 0 && KB * static_bpb<N, KIND>() >= 48;
}

// Arguments of the single-pass kernel.
struct OnepassArgs {
  const float* x;
  RowTiling rt;
  int64_t C;
  KeepMap map;
  int r, rounding;
  unsigned long long* slots;
  uint64_t tag;
  const unsigned long long* epoch;   // replayable calls: the tag is moved by *epoch
  long long wait_ticks;
  uint8_t* codes;
  int64_t pitch;
  float* scale;
};

// Body of the single-pass kernel for workgroup `bid` of `nbid` (the whole grid, or the
// leading part of a grid whose other workgroups do unrelated work).
template <int N, int VEC, int KIND, int KB>
__device__ __forceinline__ void onepass_body(const OnepassArgs& a, const int bid, const int nbid) {
  const float* __restrict__ x = a.x;
  const RowTiling rt = a.rt;
  const int64_t C = a.C;
  const KeepMap& map = a.map;
  const int r = a.r, rounding = a.rounding;
  unsigned long long* __restrict__ slots = a.slots;
  const unsigned long long tag = effective_tag(a.tag, a.epoch);
  const uint32_t tag_hi = (uint32_t)(tag >> 32), tag_lo = (uint32_t)tag;
  const long long wait_ticks = a.wait_ticks;
  uint8_t* __restrict__ codes = a.codes;
  const int64_t pitch = a.pitch;
  float* __restrict__ scale = a.scale;
  constexpr int CT = 64 * VEC;
  constexpr int BITS = KIND == kKeepAll4 ? 4 : 8;
  constexpr int QMAX = (1 << (BITS - 1)) - 1;
  extern __shared__ __align__(16) uint8_t tile[];
  __shared__ int s_nmiss;
  __shared__ uint32_t s_miss[64];   // bit b of word b/32: workgroup b's maximum did not arrive in time
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int bpb = KIND == kKeepGeneric ? r : (KIND == kKeepLowHalf ? N / 2 : (KIND == kKeepAll8 ? N : N / 2));
  const int TB = 4 * KB * bpb, TBP = TB + 4;
  const int64_t nblk = rt.nblk;
  const int64_t tiles_x = (C + CT - 1) / CT;
  const int64_t tx = bid % tiles_x, ty = bid / tiles_x;
  const int64_t c0 = tx * CT + lane * VEC;
  const bool col_ok = c0 < C;

  // Blocks one after the other, the next block's rows in flight under the current block's
  // butterflies; only the kept values stay.
  using VT = typename VecT<VEC>::type;
  constexpr int DEPTH = onepass_depth<N, VEC, KIND, KB>();
  float v[KB][VEC][kept_vals<N, KIND>()];
  float m = 0.0f;
  VT q[DEPTH][N];
  const int64_t gb0 = ty * 4 * KB + __builtin_amdgcn_readfirstlane(w) * KB;
  const float* tile_x = x + tx * CT;
  uint32_t col = (uint32_t)lane * VEC;
  // rows of block gb (clamped to a real block when gb is past the end: nothing is loaded then)
  auto issue = [&](int64_t gb, VT(&dst)[N]) {
    int64_t first;
    int valid;
    block_rows<N>(rt, gb < nblk ? gb : nblk - 1, first, valid);
    load_rows<N, VEC>(tile_x + first * C, C, col, gb < nblk && col_ok, valid, dst);
  };
  if constexpr (DEPTH == 2) issue(gb0, q[0]);
#pragma unroll
  for (int kb = 0; kb < KB; ++kb) {
    VT(&cur)[N] = q[kb % DEPTH];
    if constexpr (DEPTH == 2) {
      if (kb + 1 < KB) issue(gb0 + kb + 1, q[(kb + 1) % 2]);
    } else {
      issue(gb0 + kb, cur);
    }
    transform_kept<N, VEC, KIND>(cur, v[kb]);   // zeros for a block past the end
    m = fmaxf(m, kept_form_absmax<N, VEC, KIND>(v[kb], map));
    // Pin the order: the column offset of every later load is made to depend (through an
    // empty asm) on all finished values of this block, so the compiler can neither issue
    // all the blocks' loads up front nor postpone the butterflies, both of which spill.
#pragma unroll
    for (int vi = 0; vi < VEC; ++vi) {
      constexpr int NV = kept_vals<N, KIND>();
      static_assert(NV % 8 == 0, "kept values per column");
#pragma unroll
      for (int j = 0; j < NV; j += 8) {
        const float* t = &v[kb][vi][j];
        asm volatile("" : "+v"(col)
                     : "v"(t[0]), "v"(t[1]), "v"(t[2]), "v"(t[3]), "v"(t[4]), "v"(t[5]), "v"(t[6]),
                       "v"(t[7]));
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  m = workgroup_max(m);
  if (tid < 2)
    __hip_atomic_store(&slots[2 * bid + tid],
                       ((unsigned long long)(tid == 0 ? tag_hi : tag_lo) << 32) | __float_as_uint(m),
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (tid < 64) s_miss[tid] = 0u;
  if (tid == 0) s_nmiss = 0;
  __syncthreads();

  // collect the other workgroups' maxima, waiting a bounded time for each
  const long long t0 = wall_clock64();
  float amax = m;
  for (int b = tid; b < nbid; b += 256) {
    if (b == bid) continue;
    bool got = false;
    for (int polls = 0; polls < (1 << 16); ++polls) {   // second bound, should the clock stall
      const unsigned long long sv =
          __hip_atomic_load(&slots[2 * b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const unsigned long long sw =
          __hip_atomic_load(&slots[2 * b + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if ((uint32_t)(sv >> 32) == tag_hi && (uint32_t)(sw >> 32) == tag_lo && (uint32_t)sv == (uint32_t)sw) {
        amax = fmaxf(amax, __uint_as_float((uint32_t)sv));
        got = true;
        break;
      }
      if (wall_clock64() - t0 > wait_ticks) break;
    }
    if (!got) {
      atomicOr(&s_miss[b >> 5], 1u << (b & 31));
      atomicAdd(&s_nmiss, 1);
    }
  }
  __syncthreads();
  if (s_nmiss > 0) {   // workgroup-uniform, rare
    // Recompute the missing tiles' maxima with few registers: rows are read one (pair) at
    // a time in a rolled loop and staged in this thread's own LDS column (the code tile is
    // not in use yet), then transformed from there.
    constexpr int NS = kept_vals<N, KIND>();
    float* stage = reinterpret_cast<float*>(tile) + lane * VEC;
    for (int turn = 0; turn < 4; ++turn) {   // the four waves take turns at the staging column
      if (turn == w) {
        for (int b = 0; b < nbid; ++b) {
          if (!((s_miss[b >> 5] >> (b & 31)) & 1u)) continue;
          const int64_t btx = b % tiles_x, bty = b / tiles_x;
          const int64_t bc0 = btx * CT + lane * VEC;
          if (bc0 >= C) continue;
          for (int kb = 0; kb < KB; ++kb) {
            const int64_t gb = bty * 4 * KB + w * KB + kb;
            if (gb >= nblk) break;
            int64_t first;
            int valid;
            block_rows<N>(rt, gb, first, valid);
            const float* src = x + first * C + bc0;
            auto row = [&](int k, float (&o)[VEC]) {   // zero padding past the sample's last token
              if (k < valid) {
                unpack_vec<VEC>(*reinterpret_cast<const VT*>(src + (int64_t)k * C), o);
              } else {
#pragma unroll
                for (int vi = 0; vi < VEC; ++vi) o[vi] = 0.0f;
              }
            };
#pragma unroll 1
            for (int j = 0; j < NS; ++j) {
              float a[VEC];
              if constexpr (KIND == kKeepLowHalf) {
                float lo[VEC], hi[VEC];
                row(2 * j, lo);
                row(2 * j + 1, hi);
#pragma unroll
                for (int vi = 0; vi < VEC; ++vi) a[vi] = lo[vi] + hi[vi];
              } else {
                row(j, a);
              }
#pragma unroll
              for (int vi = 0; vi < VEC; ++vi) stage[j * 64 * VEC + vi] = a[vi];
            }
            float t[VEC][NS];
#pragma unroll
            for (int j = 0; j < NS; ++j) {
#pragma unroll
              for (int vi = 0; vi < VEC; ++vi) t[vi][j] = stage[j * 64 * VEC + vi];
            }
#pragma unroll
            for (int vi = 0; vi < VEC; ++vi) fwht_regs<NS>(t[vi]);
            amax = fmaxf(amax, kept_form_absmax<N, VEC, KIND>(t, map));
          }
        }
      }
      __syncthreads();
    }
    __syncthreads();   // staging done before the tile is zeroed / filled
  }
  amax = workgroup_max(amax);
  const float inv = quant_inv(amax, QMAX);
  if (bid == 0 && tid == 0) *scale = quant_scale(amax, QMAX);

  // A lane's codes of consecutive blocks are consecutive bytes of its column's output row:
  // with enough of them (and a compile-time kept list) they are packed in registers and leave
  // as 16-byte pieces after a wave-private transposition (or 8 bytes at a time straight from
  // registers where a run is not a multiple of 16); otherwise they go through the LDS tile.
  constexpr bool kDirect = onepass_direct_store<N, KIND, KB>();
  if constexpr (kDirect) {
    constexpr int BPB = static_bpb<N, KIND>();
    // all blocks are packed first and stored afterwards
    auto emit = [&](auto rounding_c) {
      constexpr int ROUNDING = decltype(rounding_c)::value;
      uint32_t d[KB][VEC][BPB / 4];
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
        for (int vi = 0; vi < VEC; ++vi) pack_kept_codes<N, KIND, ROUNDING>(v[kb][vi], inv, d[kb][vi]);
      }
      __builtin_amdgcn_sched_barrier(0);
      constexpr int RUN = KB * BPB;   // consecutive output bytes of a lane's column
      if constexpr (RUN % 16 == 0 && RUN >= 64) {
        // Transposed through a wave-private part of the LDS tile so that a store instruction
        // writes whole runs: the wave's codes are staged as [column][16-byte chunk] (each lane
        // its own runs), read back in linear order, and lane l of store `it` then holds chunk
        // (it * 64 + l) % CH of column (it * 64 + l) / CH: neighbouring lanes write
        // neighbouring 16 bytes of one output row (RUN bytes per row and instruction) instead
        // of 64 lanes writing 16 bytes each into 64 different rows, which left L2 as partial
        // lines (HLA of the ViT-B g_y: 35.8 -> 19.2 MB written for 19.4 MB of codes, 42 -> 38.5 us).
        // Only this wave touches the staging area and a wave's LDS instructions are performed
        // in order, so no workgroup barrier is needed.  Runs below 64 bytes keep the plain
        // stores: the extra LDS round trip costs such a short kernel more than it saves
        // (ViT-B activation, 48-byte runs: 19.0 against 17.5 us).
        constexpr int CH = RUN / 16;
        uint8_t* wt = tile + (size_t)w * (CT * RUN);
#pragma unroll
        for (int vi = 0; vi < VEC; ++vi) {
#pragma unroll
          for (int ch = 0; ch < CH; ++ch) {
            uint4 val;
            if constexpr (BPB == 8) {   // two consecutive blocks per chunk
              val = make_uint4(d[2 * ch][vi][0], d[2 * ch][vi][1], d[2 * ch + 1][vi][0], d[2 * ch + 1][vi][1]);
            } else {
              constexpr int PER = BPB / 16;   // chunks per block
              const int kb = ch / PER, dw = 4 * (ch % PER);
              val = make_uint4(d[kb][vi][dw], d[kb][vi][dw + 1], d[kb][vi][dw + 2], d[kb][vi][dw + 3]);
            }
            *reinterpret_cast<uint4*>(wt + (lane * VEC + vi) * RUN + ch * 16) = val;
          }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        uint8_t* out = codes + gb0 * BPB;
#pragma unroll
        for (int it = 0; it < VEC * CH; ++it) {
          const int f = it * 64 + lane;
          const int colw = f / CH, ch = f - colw * CH;
          const uint4 val = *reinterpret_cast<const uint4*>(wt + f * 16);
          const int64_t c = tx * CT + colw;
          // a chunk whose first block exists is stored whole: a partner block past the end
          // holds zero codes, which is what the padding up to the pitch holds anyway
          if (c < C && gb0 + (ch * 16) / BPB < nblk)
            *reinterpret_cast<uint4*>(out + c * pitch + ch * 16) = val;
        }
      } else if constexpr (BPB == 8 && KB % 2 == 0) {
        // 8-byte blocks: two consecutive blocks make one aligned 16-byte store (a wave's
        // first block is even; a partner block past the end holds zero codes, which is what
        // the padding up to the pitch holds anyway)
#pragma unroll
        for (int kb = 0; kb < KB; kb += 2) {
          const int64_t gb = ty * 4 * KB + w * KB + kb;
          if (gb < nblk && col_ok) {
#pragma unroll
            for (int vi = 0; vi < VEC; ++vi)
              *reinterpret_cast<uint4*>(codes + (c0 + vi) * pitch + gb * BPB) =
                  make_uint4(d[kb][vi][0], d[kb][vi][1], d[kb + 1][vi][0], d[kb + 1][vi][1]);
          }
        }
      } else {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
          const int slot = w * KB + kb;
          const int64_t gb = ty * 4 * KB + slot;
          if (gb < nblk && col_ok) {
#pragma unroll
            for (int vi = 0; vi < VEC; ++vi) {
              uint8_t* dst = codes + (c0 + vi) * pitch + gb * BPB;
              if constexpr (BPB % 16 == 0) {
#pragma unroll
                for (int i = 0; i < BPB / 16; ++i)
                  reinterpret_cast<uint4*>(dst)[i] = make_uint4(d[kb][vi][4 * i], d[kb][vi][4 * i + 1], d[kb][vi][4 * i + 2], d[kb][vi][4 * i + 3]);
              } else {
#pragma unroll
                for (int i = 0; i < BPB / 8; ++i)
                  reinterpret_cast<uint2*>(dst)[i] = make_uint2(d[kb][vi][2 * i], d[kb][vi][2 * i + 1]);
              }
            }
          }
        }
      }
    };
    if (rounding == 0) emit(std::integral_constant<int, 0>{});
    else emit(std::integral_constant<int, 1>{});
    // zero codes after the last block, up to the pitch (last row tile only)
    if (ty == (nblk + 4 * KB - 1) / (4 * KB) - 1) {
      const int64_t start = nblk * BPB;
      const int pad_dw = (int)((pitch - start) >> 2);
      for (int idx = tid; idx < CT * pad_dw; idx += 256) {
        const int colx = idx / pad_dw, dw = idx - colx * pad_dw;
        const int64_t c = tx * CT + colx;
        if (c < C) *reinterpret_cast<uint32_t*>(codes + c * pitch + start + 4 * dw) = 0u;
      }
    }
  } else {
    // slots of blocks past the end must read back as zero codes
    if ((ty + 1) * 4 * KB > nblk) {
      for (int i = tid; i < CT * TBP / 4; i += 256) reinterpret_cast<uint32_t*>(tile)[i] = 0u;
      __syncthreads();
    }
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
      const int slot = w * KB + kb;
      const int64_t gb = ty * 4 * KB + slot;
      if (gb < nblk && col_ok)
        store_kept_form_codes<N, VEC, KIND>(v[kb], tile, lane, slot * bpb, TBP, map, inv, rounding);
    }
    __syncthreads();
    write_out_tile<VEC>(tile, TB, TBP, tx, ty, nblk, KB, C, pitch, codes);
  }
}

template <int N, int VEC, int KIND, int KB>
__global__ __launch_bounds__(256, 2) void col_quant_onepass_kernel(const OnepassArgs a) {
  onepass_body<N, VEC, KIND, KB>(a, (int)blockIdx.x, (int)gridDim.x);
}

// Columns per lane of the single-pass kernel: two for 16-row blocks, else one.
__host__ __device__ constexpr int onepass_vec(int n) { return n == 16 ? 2 : 1; }

// Host-side launch parameters shared by the two passes.
struct ColPlan {
  int kind;
  int vec_a, kbw_a;     // abs-max pass: wide loads, few registers beyond the block itself
  int absmax_grid;
  int vec_q, kbw_q;     // quantise pass: narrow tiles, more waves in flight
  int64_t tiles_q;
  size_t lds_q;
};

ColPlan plan_col(int64_t nblk, int64_t C, int n, int r, int bits, bool lowpass_default, bool identity);

}  // namespace hot
