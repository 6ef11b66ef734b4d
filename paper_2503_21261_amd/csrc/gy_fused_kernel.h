// Both quantised views of the output gradient from two reads of g_y instead of three
// (four with a per-tensor g_x quantiser): the row-direction transform of the g_x path
// (HQ along O, Sec. 5.1) and the column-direction low-rank transform of the g_w path
// (HLA along L, Sec. 5.2) share every load.
//
// A lane owns 2 adjacent columns and holds one n-row block (n rows x 2 columns) in
// registers.  The column transform runs on a register copy (butterflies over the n
// rows); the row transform runs on the original (one in-lane butterfly, the rest
// across neighbouring lanes), so both are bit-identical to the separate kernels.
//   pass 1: HLA abs-max (partial per workgroup) and per-token abs-max partials
//           rowpart[column tile][token] (or one more partial per workgroup when the
//           g_x path quantises per tensor);
//   pass 2: both quantisations; token codes leave as dwords after a 4x4 byte transpose
//           inside lane quads, HLA codes through the LDS tile of the column kernel.
#pragma once
#include "col_quant_kernel.h"

namespace hot {

constexpr int kFusedCT = 128;   // columns per wave and per tile

// `rows` is wave-uniform (first row of the block at the tile's first column), `col` the
// lane's 32-bit column offset: the row stride is added on the scalar unit.
template <int N>
__device__ __forceinline__ void load_block_raw(const float* __restrict__ rows, int64_t C,
                                               uint32_t col, bool ok, float (&v)[2][N]) {
  float2 q[N];
#pragma unroll
  for (int k = 0; k < N; ++k)
    q[k] = ok ? *reinterpret_cast<const float2*>(rows + (int64_t)k * C + col) : make_float2(0.0f, 0.0f);
#pragma unroll
  for (int k = 0; k < N; ++k) {
    v[0][k] = q[k].x;
    v[1][k] = q[k].y;
  }
}

// Row-direction butterflies h = 1 .. N/2 for the two adjacent elements (a, b) a lane
// holds, two rows at a time; a block of N columns spans N/2 neighbouring lanes.
//
// Across lanes a butterfly is ONE instruction, own = partner * c + own with the partner read
// through a DPP permute and c = +1 in the lane that holds the lower element, -1 in the upper
// one.  The product by +-1 is exact, so the single rounding is that of the plain sum or
// difference.  The upper lane thereby computes b - a where the transform has a - b: a lane
// carries its values with the sign (-1)^(number of stages in which it was the upper lane),
// which a lane and its partner share at every stage (they differ only in the bit of that
// stage), so c stays +-1.  Magnitudes are unaffected; `flip` is the sign bit to xor into the
// reciprocal scale where the values are quantised: (sigma t) * (sigma inv) = t * inv exactly.
//
// The compiler folds a DPP permute into an add or a multiply but not into a multiply-add,
// hence the assembly.  It does not see DPP instructions inside it, so the hazards are waited
// for here: a vector write of EXEC needs 5 wait states before a DPP instruction (s_nop 4 at
// the top covers that and the 2 wait states after a vector write of a source register);
// within the block four independent chains put three instructions between a write and its
// DPP read; s_nop 1 at the end covers a DPP read the compiler may place right behind it.
template <int N>
struct LaneSigns {
  float c1, c2, c4, c8;
  uint32_t flip;
};
template <int N>
__device__ __forceinline__ LaneSigns<N> lane_signs(int lane) {
  static_assert(N == 16 || N == 32, "block size of the fused kernels");
  LaneSigns<N> s;
  s.c1 = (lane & 1) ? -1.0f : 1.0f;
  s.c2 = (lane & 2) ? -1.0f : 1.0f;
  s.c4 = (lane & 4) ? -1.0f : 1.0f;
  s.c8 = (lane & 8) ? -1.0f : 1.0f;
  s.flip = (__builtin_popcount((unsigned)lane & (N == 32 ? 15u : 7u)) & 1) ? 0x80000000u : 0u;
  return s;
}

#define HOT_DPP_ALL " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
#define HOT_FMAC4(CTRL, C)                                    \
  "v_fmac_f32_dpp %0, %0, " C " " CTRL HOT_DPP_ALL            \
  "v_fmac_f32_dpp %1, %1, " C " " CTRL HOT_DPP_ALL            \
  "v_fmac_f32_dpp %2, %2, " C " " CTRL HOT_DPP_ALL            \
  "v_fmac_f32_dpp %3, %3, " C " " CTRL HOT_DPP_ALL
// id ^ 4 and id ^ 8 are two mirrors each: the first as a move into a temporary, the second
// folded into the multiply-add
#define HOT_FMAC4_VIA(CTRL1, CTRL2, C)                        \
  "v_mov_b32_dpp %4, %0 " CTRL1 HOT_DPP_ALL                   \
  "v_mov_b32_dpp %5, %1 " CTRL1 HOT_DPP_ALL                   \
  "v_mov_b32_dpp %6, %2 " CTRL1 HOT_DPP_ALL                   \
  "v_mov_b32_dpp %7, %3 " CTRL1 HOT_DPP_ALL                   \
  "v_fmac_f32_dpp %0, %4, " C " " CTRL2 HOT_DPP_ALL           \
  "v_fmac_f32_dpp %1, %5, " C " " CTRL2 HOT_DPP_ALL           \
  "v_fmac_f32_dpp %2, %6, " C " " CTRL2 HOT_DPP_ALL           \
  "v_fmac_f32_dpp %3, %7, " C " " CTRL2 HOT_DPP_ALL

template <int N>
__device__ __forceinline__ void fwht_row2_pair(float& a0, float& b0, float& a1, float& b1,
                                               const LaneSigns<N>& s) {
  const float x0 = a0 + b0, y0 = a0 - b0;  // h = 1
  const float x1 = a1 + b1, y1 = a1 - b1;
  a0 = x0;
  b0 = y0;
  a1 = x1;
  b1 = y1;
  float t0, t1, t2, t3;
  if constexpr (N == 16) {
    asm volatile("s_nop 4\n\t"
                 HOT_FMAC4("quad_perm:[1,0,3,2]", "%8")                           // h = 2
                 HOT_FMAC4("quad_perm:[2,3,0,1]", "%9")                           // h = 4
                 HOT_FMAC4_VIA("quad_perm:[3,2,1,0]", "row_half_mirror", "%10")   // h = 8
                 "s_nop 1"
                 : "+v"(a0), "+v"(b0), "+v"(a1), "+v"(b1), "=&v"(t0), "=&v"(t1), "=&v"(t2), "=&v"(t3)
                 : "v"(s.c1), "v"(s.c2), "v"(s.c4));
  } else {
    asm volatile("s_nop 4\n\t"
                 HOT_FMAC4("quad_perm:[1,0,3,2]", "%8")                           // h = 2
                 HOT_FMAC4("quad_perm:[2,3,0,1]", "%9")                           // h = 4
                 HOT_FMAC4_VIA("quad_perm:[3,2,1,0]", "row_half_mirror", "%10")   // h = 8
                 HOT_FMAC4_VIA("row_half_mirror", "row_mirror", "%11")            // h = 16
                 "s_nop 1"
                 : "+v"(a0), "+v"(b0), "+v"(a1), "+v"(b1), "=&v"(t0), "=&v"(t1), "=&v"(t2), "=&v"(t3)
                 : "v"(s.c1), "v"(s.c2), "v"(s.c4), "v"(s.c8));
  }
}
#undef HOT_FMAC4_VIA
#undef HOT_FMAC4
#undef HOT_DPP_ALL

// One halving step of the transposing maximum: the lane keeps one half of its CNT*2
// rows and receives its partner's maxima for that half.
template <int MASK, int CNT, int N>
__device__ __forceinline__ void rows_max_step(float (&m)[N], int lane) {
  const bool up = (lane & MASK) != 0;
#pragma unroll
  for (int i = 0; i < CNT; ++i) {
    const float keep = up ? m[i + CNT] : m[i];
    const float send = up ? m[i] : m[i + CNT];
    m[i] = fmaxf(keep, lane_xor<MASK>(send));
  }
}

// m[k] = this lane's maximum for row k.  Returns the wave-wide maximum of row
// fused_row_of_lane<N>(lane); N - 1 exchanges instead of 6 N.
template <int N>
__device__ __forceinline__ float rows_max_across_lanes(float (&m)[N], int lane) {
  static_assert(N == 16 || N == 32, "block size of the fused kernels");
  rows_max_step<32, N / 2, N>(m, lane);
  rows_max_step<16, N / 4, N>(m, lane);
  rows_max_step<8, N / 8, N>(m, lane);
  rows_max_step<4, N / 16, N>(m, lane);
  if constexpr (N == 32) rows_max_step<2, 1, N>(m, lane);
  float r = m[0];
  if constexpr (N == 16) r = fmaxf(r, lane_xor<2>(r));
  return fmaxf(r, lane_xor<1>(r));
}
template <int N>
__device__ __forceinline__ int fused_row_of_lane(int lane) {
  return N == 32 ? (lane >> 1) & 31 : (lane >> 2) & 15;
}

// Pass 1.  Tiles of (4*kbw blocks) x 128 columns over a capped grid.
template <int N, int KIND, bool PER_TOKEN>
__global__ __launch_bounds__(256) void gy_fused_absmax_kernel(
    const float* __restrict__ g, int64_t L, int64_t O, KeepMap map, int kbw,
    float* __restrict__ part_hla, float* __restrict__ part_row, float* __restrict__ rowpart) {
  __shared__ float s_max[8];
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t nblk = L / N;
  const int64_t tiles_x = (O + kFusedCT - 1) / kFusedCT;
  const int64_t tiles_y = (nblk + 4 * kbw - 1) / (4 * kbw);
  const LaneSigns<N> signs = lane_signs<N>(lane);
  float mh = 0.0f, mr = 0.0f;
  for (int64_t t = blockIdx.x; t < tiles_x * tiles_y; t += gridDim.x) {
    const int64_t tx = t % tiles_x, ty = t / tiles_x;
    const int64_t c0 = tx * kFusedCT + lane * 2;
    const bool ok = c0 < O;   // lanes past the last column carry zeros through the exchanges
    for (int kb = 0; kb < kbw; ++kb) {
      const int64_t gb = ty * 4 * kbw + w * kbw + kb;
      if (gb >= nblk) break;
      float v[2][N];
      load_block_raw<N>(g + gb * N * O + tx * kFusedCT, O, (uint32_t)lane * 2u, ok, v);
      if constexpr (KIND == kKeepLowHalf) {
        float c[2][N / 2];
        fwht_even_rows<N>(v[0], c[0]);
        fwht_even_rows<N>(v[1], c[1]);
#pragma unroll
        for (int k = 0; k < N / 2; ++k) mh = fmaxf(mh, fmaxf(fabsf(c[0][k]), fabsf(c[1][k])));
      } else {
        float c[2][N];
#pragma unroll
        for (int k = 0; k < N; ++k) {
          c[0][k] = v[0][k];
          c[1][k] = v[1][k];
        }
        fwht_regs<N>(c[0]);
        fwht_regs<N>(c[1]);
#pragma unroll
        for (int k = 0; k < N; ++k)
          if (map.pos[k] >= 0) mh = fmaxf(mh, fmaxf(fabsf(c[0][k]), fabsf(c[1][k])));
      }
      float m[N];
#pragma unroll
      for (int k = 0; k < N; k += 2) {
        fwht_row2_pair<N>(v[0][k], v[1][k], v[0][k + 1], v[1][k + 1], signs);
        m[k] = fmaxf(fabsf(v[0][k]), fabsf(v[1][k]));
        m[k + 1] = fmaxf(fabsf(v[0][k + 1]), fabsf(v[1][k + 1]));
      }
      if constexpr (PER_TOKEN) {
        const float rm = rows_max_across_lanes<N>(m, lane);
        const bool writer = N == 32 ? (lane & 1) == 0 : (lane & 3) == 0;
        if (writer) rowpart[tx * L + gb * N + fused_row_of_lane<N>(lane)] = rm;
      } else {
#pragma unroll
        for (int k = 0; k < N; ++k) mr = fmaxf(mr, m[k]);
      }
    }
  }
  mh = wave_max(mh);
  mr = wave_max(mr);
  if (lane == 0) {
    s_max[w] = mh;
    s_max[4 + w] = mr;
  }
  __syncthreads();
  if (tid == 0) {
    part_hla[blockIdx.x] = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));
    if constexpr (!PER_TOKEN)
      part_row[blockIdx.x] = fmaxf(fmaxf(s_max[4], s_max[5]), fmaxf(s_max[6], s_max[7]));
  }
}

// Pass 2: one tile per workgroup.  Dynamic LDS: 4*kbw*N reciprocal token scales, then
// the HLA code tile of the column kernel (128 rows of TB + 4 bytes).
template <int N, int KIND, int BITS, bool PER_TOKEN, int ROUNDING>
__global__ __launch_bounds__(256) void gy_fused_quant_kernel(
    const float* __restrict__ g, int64_t L, int64_t O, KeepMap map, int r, int kbw,
    const float* __restrict__ part_hla, const float* __restrict__ part_row, int npartials,
    const float* __restrict__ rowpart, uint8_t* __restrict__ qg, int64_t pitch_g,
    float* __restrict__ sg, uint8_t* __restrict__ qgh, int64_t pitch_h, float* __restrict__ s_gh) {
  constexpr int QMAXG = (1 << (BITS - 1)) - 1;
  constexpr int rounding = ROUNDING;
  extern __shared__ __align__(16) uint8_t smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int rows_tile = 4 * kbw * N;
  float* s_inv = reinterpret_cast<float*>(smem);
  uint8_t* tile = smem + rows_tile * 4;
  const int bpb = KIND == kKeepGeneric ? r : N / 2;
  const int TB = 4 * kbw * bpb, TBP = TB + 4;
  const int64_t nblk = L / N;
  const int64_t tiles_x = (O + kFusedCT - 1) / kFusedCT;
  // last tile first: the first pass ended there, and the memory-side cache still holds its rows
  const int64_t bid = (int64_t)gridDim.x - 1 - blockIdx.x;
  const int64_t tx = bid % tiles_x, ty = bid / tiles_x;
  const int64_t c0 = tx * kFusedCT + lane * 2;
  const bool ok = c0 < O;
  const int64_t row0 = ty * rows_tile;
  const LaneSigns<N> signs = lane_signs<N>(lane);

  const float amax_h = block_max_of(part_hla, npartials);
  const float inv_h = quant_inv(amax_h, 127);
  if (blockIdx.x == 0 && tid == 0) *s_gh = quant_scale(amax_h, 127);
  float inv_t = 0.0f;
  if constexpr (PER_TOKEN) {
    for (int i = tid; i < rows_tile; i += 256) {
      const int64_t row = row0 + i;
      float a = 0.0f;
      if (row < L) {
        for (int64_t t = 0; t < tiles_x; ++t) a = fmaxf(a, rowpart[t * L + row]);
        if (tx == 0) sg[row] = quant_scale(a, QMAXG);
      }
      s_inv[i] = quant_inv(a, QMAXG);
    }
  } else {
    const float amax_r = block_max_of(part_row, npartials);
    inv_t = quant_inv(amax_r, QMAXG);
    if (blockIdx.x == 0 && tid == 0) sg[0] = quant_scale(amax_r, QMAXG);
  }
  // slots of blocks past the end must read back as zero codes
  if ((ty + 1) * 4 * kbw > nblk)
    for (int i = tid; i < kFusedCT * TBP / 4; i += 256) reinterpret_cast<uint32_t*>(tile)[i] = 0u;
  __syncthreads();

  for (int kb = 0; kb < kbw; ++kb) {
    const int slot = w * kbw + kb;
    const int64_t gb = ty * 4 * kbw + slot;
    if (gb >= nblk) continue;
    float v[2][N];
    load_block_raw<N>(g + gb * N * O + tx * kFusedCT, O, (uint32_t)lane * 2u, ok, v);
    if constexpr (KIND == kKeepLowHalf) {
      float c[2][N / 2];
      fwht_even_rows<N>(v[0], c[0]);
      fwht_even_rows<N>(v[1], c[1]);
#pragma unroll
      for (int vi = 0; vi < 2; ++vi) {
        uint32_t* dst = reinterpret_cast<uint32_t*>(tile + (vi * 64 + lane) * TBP + slot * bpb);
#pragma unroll
        for (int j4 = 0; j4 < N / 8; ++j4) {
          int q[4];
#pragma unroll
          for (int e = 0; e < 4; ++e)   // even natural row 2k' sits at c[k']
            q[e] = quant_code(c[vi][lowpass_row(N, j4 * 4 + e) >> 1], inv_h, 127, rounding);
          dst[j4] = pack4_codes8(q[0], q[1], q[2], q[3]);
        }
      }
    } else {
      float c[2][N];
#pragma unroll
      for (int k = 0; k < N; ++k) {
        c[0][k] = v[0][k];
        c[1][k] = v[1][k];
      }
      fwht_regs<N>(c[0]);
      fwht_regs<N>(c[1]);
      store_block_codes<N, 2, KIND>(c, tile, lane, slot * bpb, TBP, map, inv_h, rounding);
    }
    if constexpr (BITS == 4) {
      // a byte per lane and row; 4 rows x 4 lanes of a quad -> one dword per lane
      const int q = lane & 3;
      const uint32_t sel_a = (q & 1) ? 0x03070105u : 0x06020400u;
      const uint32_t sel_b = (q & 2) ? 0x03020706u : 0x05040100u;
      uint8_t* dst = qg + (gb * N + q) * pitch_g + tx * (kFusedCT / 2) + 4 * (lane >> 2);
#pragma unroll
      for (int k4 = 0; k4 < N / 4; ++k4) {
        uint32_t word = 0;
        fwht_row2_pair<N>(v[0][4 * k4], v[1][4 * k4], v[0][4 * k4 + 1], v[1][4 * k4 + 1], signs);
        fwht_row2_pair<N>(v[0][4 * k4 + 2], v[1][4 * k4 + 2], v[0][4 * k4 + 3], v[1][4 * k4 + 3], signs);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int k = 4 * k4 + e;
          const float inv = __uint_as_float(__float_as_uint(PER_TOKEN ? s_inv[slot * N + k] : inv_t) ^ signs.flip);
          const int a = quant_code(v[0][k], inv, QMAXG, rounding);
          const int b = quant_code(v[1][k], inv, QMAXG, rounding);
          word |= (uint32_t)((a & 0xF) | ((b & 0xF) << 4)) << (8 * e);
        }
        const uint32_t p1 = (uint32_t)__builtin_amdgcn_mov_dpp((int)word, 0xB1, 0xF, 0xF, true);
        const uint32_t half = __builtin_amdgcn_perm(p1, word, sel_a);
        const uint32_t p2 = (uint32_t)__builtin_amdgcn_mov_dpp((int)half, 0x4E, 0xF, 0xF, true);
        const uint32_t full = __builtin_amdgcn_perm(p2, half, sel_b);
        if (ok) *reinterpret_cast<uint32_t*>(dst + (int64_t)(4 * k4) * pitch_g) = full;
      }
    } else {
      // two bytes per lane and row; 2 rows x 2 lanes -> one dword per lane
      const int q = lane & 1;
      const uint32_t sel = q ? 0x03020706u : 0x05040100u;
      uint8_t* dst = qg + (gb * N + q) * pitch_g + tx * kFusedCT + 4 * (lane >> 1);
#pragma unroll
      for (int k2 = 0; k2 < N / 2; ++k2) {
        uint32_t word = 0;
        fwht_row2_pair<N>(v[0][2 * k2], v[1][2 * k2], v[0][2 * k2 + 1], v[1][2 * k2 + 1], signs);
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const int k = 2 * k2 + e;
          const float inv = __uint_as_float(__float_as_uint(PER_TOKEN ? s_inv[slot * N + k] : inv_t) ^ signs.flip);
          const int a = quant_code(v[0][k], inv, QMAXG, rounding);
          const int b = quant_code(v[1][k], inv, QMAXG, rounding);
          word |= (uint32_t)((a & 0xFF) | ((b & 0xFF) << 8)) << (16 * e);
        }
        const uint32_t p1 = (uint32_t)__builtin_amdgcn_mov_dpp((int)word, 0xB1, 0xF, 0xF, true);
        const uint32_t full = __builtin_amdgcn_perm(p1, word, sel);
        if (ok) *reinterpret_cast<uint32_t*>(dst + (int64_t)(2 * k2) * pitch_g) = full;
      }
    }
  }

  // zero codes from the last column up to the pitch of the token rows
  if (tx == tiles_x - 1) {
    const int64_t ob = O * BITS / 8;
    const int pad_dw = (int)((pitch_g - ob) >> 2);
    for (int idx = tid; idx < rows_tile * pad_dw; idx += 256) {
      const int i = idx / pad_dw, dw = idx - i * pad_dw;
      if (row0 + i < L) *reinterpret_cast<uint32_t*>(qg + (row0 + i) * pitch_g + ob + 4 * dw) = 0u;
    }
  }
  __syncthreads();
  write_out_tile<2>(tile, TB, TBP, tx, ty, nblk, kbw, O, pitch_h, qgh);
}

}  // namespace hot
