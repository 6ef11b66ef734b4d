// Device-side helpers shared by the HOT kernels (gfx950 only, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hot {

constexpr int kWave = 64;

// ---- cross-lane exchange: value held by lane (id ^ MASK) -------------------
// MASK 1..8 are DPP permutes on the vector pipe (4 and 8 as two mirrors: reversing 4
// then 8 lanes exchanges the halves of every 8, reversing 8 then 16 those of every 16);
// 16 uses the ds_swizzle bit mode (no LDS memory is touched), 32 swaps the wave halves.
template <int MASK>
__device__ __forceinline__ float lane_xor(float v) {
  int x = __float_as_int(v);
  int r;
  if constexpr (MASK == 1) {
    r = __builtin_amdgcn_mov_dpp(x, 0xB1, 0xF, 0xF, true);   // quad_perm [1,0,3,2]
  } else if constexpr (MASK == 2) {
    r = __builtin_amdgcn_mov_dpp(x, 0x4E, 0xF, 0xF, true);   // quad_perm [2,3,0,1]
  } else if constexpr (MASK == 4) {
    const int t = __builtin_amdgcn_mov_dpp(x, 0x1B, 0xF, 0xF, true);   // quad_perm [3,2,1,0]
    r = __builtin_amdgcn_mov_dpp(t, 0x141, 0xF, 0xF, true);            // row_half_mirror
  } else if constexpr (MASK == 8) {
    const int t = __builtin_amdgcn_mov_dpp(x, 0x141, 0xF, 0xF, true);  // row_half_mirror
    r = __builtin_amdgcn_mov_dpp(t, 0x140, 0xF, 0xF, true);            // row_mirror
  } else if constexpr (MASK == 16) {
    r = __builtin_amdgcn_ds_swizzle(x, (MASK << 10) | 0x1F); // and 0x1F, or 0, xor MASK
  } else {
    static_assert(MASK == 32, "lane_xor mask");
    r = __builtin_amdgcn_ds_bpermute(((int)(threadIdx.x & 63) ^ 32) << 2, x);
  }
  return __int_as_float(r);
}

// Launch tag of a kernel whose workgroups exchange values through the workspace: the host's
// per-launch tag, or, in a replayable call, that tag moved by the workspace epoch which every
// such call advances first (a replayed graph repeats the host's tag but not the epoch).
__device__ __forceinline__ unsigned long long effective_tag(unsigned long long host_tag,
                                                            const unsigned long long* epoch) {
  if (!epoch) return host_tag;
  const unsigned long long t = host_tag + *epoch * 0x9E3779B97F4A7C15ull;
  return t ? t : 1ull;   // zero is never a tag
}

__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, lane_xor<1>(v));
  v = fmaxf(v, lane_xor<2>(v));
  v = fmaxf(v, lane_xor<4>(v));
  v = fmaxf(v, lane_xor<8>(v));
  v = fmaxf(v, lane_xor<16>(v));
  v = fmaxf(v, lane_xor<32>(v));
  return v;
}

// One butterfly stage across lanes: the lane whose MASK bit is clear holds the
// lower element a, its partner the upper element b; (a, b) -> (a + b, a - b).
// The upper lane adds its own value with the sign flipped: p + (-v) is p - v exactly.
template <int MASK>
__device__ __forceinline__ float butterfly_lanes(float v, bool upper) {
  const float p = lane_xor<MASK>(v);
  const float s = __int_as_float(__float_as_int(v) ^ (upper ? (int)0x80000000 : 0));
  return p + s;
}

// In-register Walsh-Hadamard butterflies of a length-N array (Sec. 3.1), stages
// h = 1, 2, 4, ... in that order: element j with bit h clear pairs with j + h.
template <int N>
__device__ __forceinline__ void fwht_regs(float (&v)[N]) {
#pragma unroll
  for (int h = 1; h < N; h *= 2) {
#pragma unroll
    for (int j = 0; j < N; ++j) {
      if ((j & h) == 0) {
        float a = v[j], b = v[j + h];
        v[j] = a + b;
        v[j + h] = a - b;
      }
    }
  }
}

// Stages h = 1 .. N/2 of the transform for the 4 elements this lane holds;
// `lane` is the lane's index within the row (its low bits select the block half).
template <int N>
__device__ __forceinline__ void fwht_row4(float4& q, int lane) {
  float x = q.x + q.y, y = q.x - q.y, z = q.z + q.w, w = q.z - q.w;  // h = 1
  q.x = x + z; q.z = x - z; q.y = y + w; q.w = y - w;                // h = 2
#define HOT_STAGE(MASK)                                      \
  {                                                          \
    const bool up = (lane & MASK) != 0;                      \
    q.x = butterfly_lanes<MASK>(q.x, up);                    \
    q.y = butterfly_lanes<MASK>(q.y, up);                    \
    q.z = butterfly_lanes<MASK>(q.z, up);                    \
    q.w = butterfly_lanes<MASK>(q.w, up);                    \
  }
  HOT_STAGE(1)  // h = 4
  HOT_STAGE(2)  // h = 8
  if constexpr (N >= 32) HOT_STAGE(4)   // h = 16
  if constexpr (N >= 64) HOT_STAGE(8)   // h = 32
#undef HOT_STAGE
}

__device__ __forceinline__ float absmax4(const float4& q) {
  return fmaxf(fmaxf(fabsf(q.x), fabsf(q.y)), fmaxf(fabsf(q.z), fabsf(q.w)));
}

// ---- quantiser (Sec. 5.1) ---------------------------------------------------
// scale = amax / qmax, inv = qmax / amax (IEEE fp32 divisions), 0 for a zero group.
__device__ __forceinline__ float quant_scale(float amax, int qmax) { return amax / (float)qmax; }
__device__ __forceinline__ float quant_inv(float amax, int qmax) {
  return amax > 0.0f ? (float)qmax / amax : 0.0f;
}

// code = clamp(round(t * inv)); pseudo-stochastic rounding compares the fractional
// part with the low 11 bits of the scaled value's own fp32 pattern, as a fraction.
__device__ __forceinline__ int quant_code(float t, float inv, int qmax, int rounding) {
  float v = t * inv;
  int q;
  if (rounding == 0) {
    q = (int)rintf(v);
  } else {
    float f = floorf(v);
    float frac = v - f;
    float rnd = (float)(__float_as_uint(v) & 0x7FFu) * (1.0f / 2048.0f);
    q = (int)f + (frac > rnd ? 1 : 0);
  }
  return min(max(q, -qmax), qmax);
}

// Four int8 codes (the low byte of each int) as one dword, c0 in byte 0: three byte
// permutes instead of a mask, a shift and an or per code.
__device__ __forceinline__ uint32_t pack4_codes8(int c0, int c1, int c2, int c3) {
  const uint32_t lo = __builtin_amdgcn_perm((uint32_t)c1, (uint32_t)c0, 0x0c0c0400u);
  const uint32_t hi = __builtin_amdgcn_perm((uint32_t)c3, (uint32_t)c2, 0x0c0c0400u);
  return __builtin_amdgcn_perm(hi, lo, 0x05040100u);
}

// Eight int4 codes (the low nibble of each int) as one dword, c[0] in the lowest nibble.
__device__ __forceinline__ uint32_t pack8_codes4(const int (&c)[8]) {
  int b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) b[i] = (c[2 * i] & 0xF) | (c[2 * i + 1] << 4);   // byte 0 is what counts
  return pack4_codes8(b[0], b[1], b[2], b[3]);
}

// Maximum of partials[0..count), returned to every thread of a 256-thread workgroup.
// The abs-max kernels leave one partial per workgroup; their consumers call this
// first, so no atomics and no pre-zeroed memory are involved.
__device__ __forceinline__ float block_max_of(const float* __restrict__ partials, int count) {
  __shared__ float s_part[4];
  float m = 0.0f;
  for (int i = threadIdx.x; i < count; i += 256) m = fmaxf(m, partials[i]);
  m = wave_max(m);
  if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = m;
  __syncthreads();
  m = fmaxf(fmaxf(s_part[0], s_part[1]), fmaxf(s_part[2], s_part[3]));
  __syncthreads();
  return m;
}

}  // namespace hot
