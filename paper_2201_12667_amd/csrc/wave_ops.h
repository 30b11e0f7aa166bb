// Cross-lane primitives of a 64-lane wavefront built on DPP moves (register-to-register, a few
// cycles each) instead of ds_bpermute shuffles (an LDS round trip each).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace slide {

// DPP controls of gfx9-family targets.
constexpr int kDppQuadSwap1 = 0xB1;      // quad_perm:[1,0,3,2]
constexpr int kDppQuadSwap2 = 0x4E;      // quad_perm:[2,3,0,1]
constexpr int kDppRowShr = 0x110;        // + n: lane i reads lane i-n of its 16-lane row
constexpr int kDppRowRor = 0x120;        // + n: lane i reads lane (i - n) mod 16 of its row
constexpr int kDppRowMirror = 0x140;     // lane i reads lane 15-i of its row
constexpr int kDppRowHalfMirror = 0x141; // lane i reads lane 7-i of its half row
constexpr int kDppRowBcast15 = 0x142;    // lane 15 of each row to the whole next row
constexpr int kDppRowBcast31 = 0x143;    // lane 31 to rows 2 and 3

// Lanes whose source is out of range (or masked off by row_mask) receive `identity`.
template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t identity, uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)identity, (int)v, CTRL, ROW_MASK, 0xf, false);
}
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}

// Inclusive prefix sum over the 16-lane rows.
__device__ __forceinline__ uint32_t row_incl_scan_add(uint32_t v) {
  v += dpp_u32<kDppRowShr + 1>(0u, v);
  v += dpp_u32<kDppRowShr + 2>(0u, v);
  v += dpp_u32<kDppRowShr + 4>(0u, v);
  v += dpp_u32<kDppRowShr + 8>(0u, v);
  return v;
}
// Inclusive prefix sum over each 32-lane half of the wave.
__device__ __forceinline__ uint32_t half_incl_scan_add(uint32_t v) {
  v = row_incl_scan_add(v);
  v += dpp_u32<kDppRowBcast15, 0xa>(0u, v);
  return v;
}
// Inclusive prefix sum over the wave.
__device__ __forceinline__ uint32_t wave_incl_scan_add(uint32_t v) {
  v = half_incl_scan_add(v);
  v += dpp_u32<kDppRowBcast31, 0xc>(0u, v);
  return v;
}
// Sum over the wave, returned in every lane (wave-uniform).
__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_readlane((int)wave_incl_scan_add(v), 63);
}
__device__ __forceinline__ uint32_t wave_or(uint32_t v) {
  v |= dpp_u32<kDppRowShr + 1>(0u, v);
  v |= dpp_u32<kDppRowShr + 2>(0u, v);
  v |= dpp_u32<kDppRowShr + 4>(0u, v);
  v |= dpp_u32<kDppRowShr + 8>(0u, v);
  v |= dpp_u32<kDppRowBcast15, 0xa>(0u, v);
  v |= dpp_u32<kDppRowBcast31, 0xc>(0u, v);
  return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// Inclusive prefix sum over aligned groups of G consecutive lanes (G a power of two <= 64).
__device__ __forceinline__ uint32_t group_incl_scan_add(uint32_t v, int G) {
  if (G == 64) return wave_incl_scan_add(v);
  if (G == 32) return half_incl_scan_add(v);
  if (G == 16) return row_incl_scan_add(v);
  const int lane = threadIdx.x & 63;
  for (int d = 1; d < G; d <<= 1) {
    const uint32_t t = __shfl_up(v, d, G);
    if ((lane & (G - 1)) >= d) v += t;
  }
  return v;
}
// The same for G <= 8 (1, 2, 4 or 8), in register moves only.
__device__ __forceinline__ uint32_t small_group_incl_scan_add(uint32_t v, int G) {
  const int p = threadIdx.x & (G - 1);
  uint32_t t = dpp_u32<kDppRowShr + 1>(0u, v);
  if (p >= 1) v += t;
  t = dpp_u32<kDppRowShr + 2>(0u, v);
  if (p >= 2) v += t;
  t = dpp_u32<kDppRowShr + 4>(0u, v);
  if (p >= 4) v += t;
  return v;
}
// Sum over aligned groups of G lanes, valid in the LAST lane of each group.
__device__ __forceinline__ uint32_t group_sum_last(uint32_t v, int G) { return group_incl_scan_add(v, G); }

// Number of the other 15 lanes of the 16-lane row whose value is smaller (values distinct within a
// row, up to repeated padding values that no lane uses): the lane's rank in the row's order.
__device__ __forceinline__ uint32_t row_rank_i32(int32_t v) {
  uint32_t r = 0;
#define SLIDE_ROR(n) r += (int32_t)dpp_u32<kDppRowRor + n>(0u, (uint32_t)v) < v ? 1u : 0u;
  SLIDE_ROR(1) SLIDE_ROR(2) SLIDE_ROR(3) SLIDE_ROR(4) SLIDE_ROR(5) SLIDE_ROR(6) SLIDE_ROR(7) SLIDE_ROR(8)
  SLIDE_ROR(9) SLIDE_ROR(10) SLIDE_ROR(11) SLIDE_ROR(12) SLIDE_ROR(13) SLIDE_ROR(14) SLIDE_ROR(15)
#undef SLIDE_ROR
  return r;
}

// Sum over aligned groups of 8 / 16 lanes, returned in every lane of the group.
__device__ __forceinline__ float sum8(float v) {
  v += dpp_f32<kDppQuadSwap1>(v);
  v += dpp_f32<kDppQuadSwap2>(v);
  v += dpp_f32<kDppRowHalfMirror>(v);
  return v;
}
__device__ __forceinline__ float sum16(float v) {
  v = sum8(v);
  v += dpp_f32<kDppRowMirror>(v);
  return v;
}
// Sum over aligned groups of LPR lanes (8, 16, 32 or 64), returned in every lane of the group.
template <int LPR>
__device__ __forceinline__ float group_sum(float v) {
  if (LPR == 8) return sum8(v);
  v = sum16(v);
  if (LPR >= 32) v += __shfl_xor(v, 16);
  if (LPR >= 64) v += __shfl_xor(v, 32);
  return v;
}

}  // namespace slide
