// Cross-lane data movement for 64-wide wavefronts on gfx950, for 64-bit values.
//
// lane_xor<MASK>(v) returns v of lane (lane ^ MASK).  Every mask used by the kernels maps to the
// cheapest mechanism the hardware has for it:
//   1, 2, 3   DPP quad_perm          7   DPP row_half_mirror      15  DPP row_mirror
//   8         DPP row_ror:8          other masks below 32: ds_swizzle in bit-mask mode (LDS crossbar,
//   no LDS memory), 32: v_permlane32_swap, above 32: the two combined.
// DPP moves run on the vector ALU at 32-bit rate; ds_bpermute-based shuffles cost about four times as
// much per 64-bit value and are not used.
#pragma once
#include <hip/hip_runtime.h>

namespace tsenor_dev {

constexpr int kWave = 64;

template <int CTRL>
__device__ __forceinline__ double dpp_mov(double v) {
  const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xF, 0xF, true);
  const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xF, 0xF, true);
  return __hiloint2double(hi, lo);
}

template <int MASK>
__device__ __forceinline__ double lane_xor(double v) {
  static_assert(MASK > 0 && MASK < kWave, "lane mask");
  if constexpr (MASK == 1) {
    return dpp_mov<0xB1>(v);  // quad_perm [1,0,3,2]
  } else if constexpr (MASK == 2) {
    return dpp_mov<0x4E>(v);  // quad_perm [2,3,0,1]
  } else if constexpr (MASK == 3) {
    return dpp_mov<0x1B>(v);  // quad_perm [3,2,1,0]
  } else if constexpr (MASK == 7) {
    return dpp_mov<0x141>(v);  // row_half_mirror
  } else if constexpr (MASK == 15) {
    return dpp_mov<0x140>(v);  // row_mirror
  } else if constexpr (MASK == 8) {
    return dpp_mov<0x128>(v);  // row_ror:8
  } else if constexpr (MASK < 32) {
    constexpr int pattern = (MASK << 10) | 0x1F;  // bit-mask mode: and 0x1F, or 0, xor MASK
    const int lo = __builtin_amdgcn_ds_swizzle(__double2loint(v), pattern);
    const int hi = __builtin_amdgcn_ds_swizzle(__double2hiint(v), pattern);
    return __hiloint2double(hi, lo);
  } else if constexpr (MASK == 32) {
    const unsigned lo = (unsigned)__double2loint(v), hi = (unsigned)__double2hiint(v);
    // swaps lanes 32..63 of the first operand with lanes 0..31 of the second
    const auto rl = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
    const auto rh = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
    const bool upper = (__lane_id() & 32) != 0;
    return __hiloint2double((int)(upper ? rh[0] : rh[1]), (int)(upper ? rl[0] : rl[1]));
  } else {
    return lane_xor<32>(lane_xor<(MASK & 31)>(v));
  }
}

// 32-bit variant of lane_xor
template <int MASK>
__device__ __forceinline__ int lane_xor_i32(int v) {
  static_assert(MASK > 0 && MASK < kWave, "lane mask");
  if constexpr (MASK == 1) {
    return __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, true);
  } else if constexpr (MASK == 2) {
    return __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, true);
  } else if constexpr (MASK == 3) {
    return __builtin_amdgcn_update_dpp(0, v, 0x1B, 0xF, 0xF, true);
  } else if constexpr (MASK == 7) {
    return __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, true);
  } else if constexpr (MASK == 15) {
    return __builtin_amdgcn_update_dpp(0, v, 0x140, 0xF, 0xF, true);
  } else if constexpr (MASK == 8) {
    return __builtin_amdgcn_update_dpp(0, v, 0x128, 0xF, 0xF, true);
  } else if constexpr (MASK < 32) {
    return __builtin_amdgcn_ds_swizzle(v, (MASK << 10) | 0x1F);
  } else if constexpr (MASK == 32) {
    const auto r = __builtin_amdgcn_permlane32_swap((unsigned)v, (unsigned)v, false, false);
    return (int)((__lane_id() & 32) ? r[0] : r[1]);
  } else {
    return lane_xor_i32<32>(lane_xor_i32<(MASK & 31)>(v));
  }
}

// max over the lanes of a group of LPB consecutive lanes (LPB a power of two)
template <int LPB, int STEP = 1>
__device__ __forceinline__ double group_max(double v) {
  if constexpr (STEP < LPB) {
    v = fmax(v, lane_xor<STEP>(v));
    return group_max<LPB, STEP * 2>(v);
  } else {
    return v;
  }
}

}  // namespace tsenor_dev
