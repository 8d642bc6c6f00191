// Small per-lane building blocks shared by the bandwidth-bound kernels: 16-bit dot products
// with fp32 accumulation and sums across lanes on the DPP path of the vector ALU.
#pragma once
#include "ap_common.hpp"

namespace ap {

typedef _Float16 h2_t __attribute__((ext_vector_type(2)));
typedef __bf16 b2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c, F16Tag) {
  return __builtin_amdgcn_fdot2(__builtin_bit_cast(h2_t, a), __builtin_bit_cast(h2_t, b), c, false);
}
__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c, BF16Tag) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(b2_t, a), __builtin_bit_cast(b2_t, b), c,
                                         false);
}
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
constexpr float kLn2 = 0.6931471805599453f;

template <class Tag>
__device__ __forceinline__ float dot8(const u32x4_t& a, const u32x4_t& b, float c) {
#pragma unroll
  for (int e = 0; e < 4; ++e) c = dot2(a[e], b[e], c, Tag{});
  return c;
}

// Lane-crossing sums on the DPP path of the vector ALU (no LDS traffic).  dpp_add<CTRL> is
// x + x[permuted]; written with a zero fill value and bound_ctrl so that the compiler folds
// the permutation into the add itself.
template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ float dpp_add(float x) {
  const int v = __builtin_bit_cast(int, x);
  return x + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xf, true));
}
// Sum over groups of N consecutive lanes (N = 2, 4, 8, 16 or 32), every lane of a group
// receiving the total: butterflies inside a 16-lane row, one shuffle across rows.
template <int N>
__device__ __forceinline__ float group_sum(float x) {
  x = dpp_add<0xB1>(x);                  // quad_perm [1,0,3,2]
  if (N >= 4) x = dpp_add<0x4E>(x);      // quad_perm [2,3,0,1]
  if (N >= 8) x = dpp_add<0x141>(x);     // row_half_mirror: the other quad of an 8-lane group
  if (N >= 16) x = dpp_add<0x140>(x);    // row_mirror: the other half of the row
  if (N >= 32) x += __shfl_xor(x, 16);
  return x;
}
// The value held by the other half of a group of N consecutive lanes (N = 4, 8, 16 or 32), for
// values that are uniform inside each half: lane i reads its mirror image in the group.
template <int N>
__device__ __forceinline__ float other_half(float x) {
  const int v = __builtin_bit_cast(int, x);
  if (N == 4) return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xf, 0xf, true));
  if (N == 8) return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, v, 0x141, 0xf, 0xf, true));
  if (N == 16) return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, v, 0x140, 0xf, 0xf, true));
  return __shfl_xor(x, 16);
}
// Sum over the 64 lanes, returned wave-uniform: row totals, then rows 1 and 3 take the
// previous row's total (row_bcast15), then rows 2 and 3 take lane 31's (row_bcast31); lane 63
// ends with everything.
__device__ __forceinline__ float wave_sum(float x) {
  x = group_sum<16>(x);
  x = dpp_add<0x142, 0xa>(x);
  x = dpp_add<0x143, 0xc>(x);
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 63));
}

}  // namespace ap
