// Wave-wide reductions and scans on the vector ALU's data-parallel-primitive (DPP) lane routing:
// no LDS crossbar traffic, a few cycles per level instead of a shuffle's LDS round trip.
// A wave is 4 DPP rows of 16 lanes.  Lanes whose source falls outside their row (shifts) or that
// the row mask leaves out keep the `old` operand, which every helper sets to the operation's
// identity.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fkv {

constexpr int kDppRowShr = 0x110;   // + n: lane i reads lane i - n of its row
constexpr int kDppRowRor = 0x120;   // + n: lane i reads lane (i - n) mod 16 of its row
constexpr int kDppBcast15 = 0x142;  // lane 15 of each row to every lane of the next row
constexpr int kDppBcast31 = 0x143;  // lane 31 to every lane of rows 2 and 3

template <int kCtrl, int kRowMask = 0xF>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t old, uint32_t src) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)old, (int)src, kCtrl, kRowMask, 0xF, false);
}

// Inclusive prefix sum over the 64 lanes (lane order).
__device__ __forceinline__ uint32_t wave_scan_add(uint32_t x) {
  x += dpp_u32<kDppRowShr + 1>(0u, x);
  x += dpp_u32<kDppRowShr + 2>(0u, x);
  x += dpp_u32<kDppRowShr + 4>(0u, x);
  x += dpp_u32<kDppRowShr + 8>(0u, x);
  x += dpp_u32<kDppBcast15, 0xA>(0u, x);  // rows 1, 3 += total of the row before
  x += dpp_u32<kDppBcast31, 0xC>(0u, x);  // rows 2, 3 += total of rows 0..1
  return x;
}

// Value of lane 63 as a wave-uniform scalar.
__device__ __forceinline__ uint32_t wave_last(uint32_t x) { return (uint32_t)__builtin_amdgcn_readlane((int)x, 63); }

// Maximum / minimum over the 64 lanes; the result is valid in lane 63 only (use wave_last to spread it).
__device__ __forceinline__ uint32_t wave_max_to_last(uint32_t x) {
  x = max(x, dpp_u32<kDppRowRor + 8>(x, x));
  x = max(x, dpp_u32<kDppRowRor + 4>(x, x));
  x = max(x, dpp_u32<kDppRowRor + 2>(x, x));
  x = max(x, dpp_u32<kDppRowRor + 1>(x, x));
  x = max(x, dpp_u32<kDppBcast15, 0xA>(x, x));
  x = max(x, dpp_u32<kDppBcast31, 0xC>(x, x));
  return x;
}
__device__ __forceinline__ uint32_t wave_min_to_last(uint32_t x) { return ~wave_max_to_last(~x); }

// Sum over the 64 lanes, valid in lane 63 only.
__device__ __forceinline__ uint32_t wave_sum_to_last(uint32_t x) {
  x += dpp_u32<kDppRowRor + 8>(0u, x);
  x += dpp_u32<kDppRowRor + 4>(0u, x);
  x += dpp_u32<kDppRowRor + 2>(0u, x);
  x += dpp_u32<kDppRowRor + 1>(0u, x);
  x += dpp_u32<kDppBcast15, 0xA>(0u, x);
  x += dpp_u32<kDppBcast31, 0xC>(0u, x);
  return x;
}

// ---- fp32 variants --------------------------------------------------------------------------
template <int kCtrl, int kRowMask = 0xF>
__device__ __forceinline__ float dpp_f32(float old, float src) {
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(old), __float_as_int(src), kCtrl, kRowMask, 0xF, false));
}

// Maximum / sum over the 32 lanes of each wave half (lanes 0-31 and 32-63 separately), in every lane.
// Rotations inside the 16-lane DPP rows, then one swap of the odd and even rows.  The summation order
// depends on the lane, so two lanes of a half may differ in the last bit: callers that need one
// value take it from a fixed lane.
__device__ __forceinline__ float half_max(float x) {
  x = fmaxf(x, dpp_f32<kDppRowRor + 8>(x, x));
  x = fmaxf(x, dpp_f32<kDppRowRor + 4>(x, x));
  x = fmaxf(x, dpp_f32<kDppRowRor + 2>(x, x));
  x = fmaxf(x, dpp_f32<kDppRowRor + 1>(x, x));
  const unsigned u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_sum(float x) {
  x += dpp_f32<kDppRowRor + 8>(0.f, x);
  x += dpp_f32<kDppRowRor + 4>(0.f, x);
  x += dpp_f32<kDppRowRor + 2>(0.f, x);
  x += dpp_f32<kDppRowRor + 1>(0.f, x);
  const unsigned u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Maximum / sum over the 64 lanes as a wave-uniform value (fixed order: reproducible).
__device__ __forceinline__ float wave_fmax(float x) {
  x = fmaxf(x, dpp_f32<kDppRowRor + 8>(x, x));
  x = fmaxf(x, dpp_f32<kDppRowRor + 4>(x, x));
  x = fmaxf(x, dpp_f32<kDppRowRor + 2>(x, x));
  x = fmaxf(x, dpp_f32<kDppRowRor + 1>(x, x));
  x = fmaxf(x, dpp_f32<kDppBcast15, 0xA>(x, x));
  x = fmaxf(x, dpp_f32<kDppBcast31, 0xC>(x, x));
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}
__device__ __forceinline__ float wave_fsum(float x) {
  x += dpp_f32<kDppRowRor + 8>(0.f, x);
  x += dpp_f32<kDppRowRor + 4>(0.f, x);
  x += dpp_f32<kDppRowRor + 2>(0.f, x);
  x += dpp_f32<kDppRowRor + 1>(0.f, x);
  x += dpp_f32<kDppBcast15, 0xA>(0.f, x);
  x += dpp_f32<kDppBcast31, 0xC>(0.f, x);
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}

}  // namespace fkv
