// Cross-lane data movement for 64-wide wavefronts on gfx950, for 64-bit values.
//
// lane_xor<MASK>(v) returns v of lane (lane ^ MASK).  Every mask used by the kernels maps to the
// cheapest mechanism the hardware has for it:
//   1, 2, 3   DPP quad_perm          7   DPP row_half_mirror      15  DPP row_mirror
//   8         DPP row_ror:8          4   two bank-masked DPP row shifts
//   16        v_permlane16_swap      32  v_permlane32_swap        larger masks: compositions of these
// All of these run on the vector ALU with a few cycles of latency.  ds_swizzle (the fallback for masks
// not listed) and ds_bpermute-based shuffles go through the LDS pipeline: ~100 cycles of latency per
// exchange, which a kernel with two waves per SIMD cannot hide in its reduction chains.
#pragma once
#include <hip/hip_runtime.h>

namespace tsenor_dev {

constexpr int kWave = 64;

// 32-bit value of lane (lane ^ MASK)
template <int MASK>
__device__ __forceinline__ int lane_xor_i32(int v) {
  static_assert(MASK > 0 && MASK < kWave, "lane mask");
  if constexpr (MASK == 1) {
    return __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, true);  // quad_perm [1,0,3,2]
  } else if constexpr (MASK == 2) {
    return __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, true);  // quad_perm [2,3,0,1]
  } else if constexpr (MASK == 3) {
    return __builtin_amdgcn_update_dpp(0, v, 0x1B, 0xF, 0xF, true);  // quad_perm [3,2,1,0]
  } else if constexpr (MASK == 7) {
    return __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, true);  // row_half_mirror
  } else if constexpr (MASK == 15) {
    return __builtin_amdgcn_update_dpp(0, v, 0x140, 0xF, 0xF, true);  // row_mirror
  } else if constexpr (MASK == 8) {
    return __builtin_amdgcn_update_dpp(0, v, 0x128, 0xF, 0xF, true);  // row_ror:8
  } else if constexpr (MASK == 4) {
    // banks 0 and 2 (lanes 0-3, 8-11 of a row) read four lanes up, banks 1 and 3 four lanes down
    const int up = __builtin_amdgcn_update_dpp(0, v, 0x104, 0xF, 0x5, false);  // row_shl:4
    return __builtin_amdgcn_update_dpp(up, v, 0x114, 0xF, 0xA, false);        // row_shr:4
  } else if constexpr (MASK == 16) {
    // swaps the odd 16-lane rows of the first operand with the even rows of the second
    const auto r = __builtin_amdgcn_permlane16_swap((unsigned)v, (unsigned)v, false, false);
    return (int)((__lane_id() & 16) ? r[0] : r[1]);
  } else if constexpr (MASK == 32) {
    // swaps lanes 32..63 of the first operand with lanes 0..31 of the second
    const auto r = __builtin_amdgcn_permlane32_swap((unsigned)v, (unsigned)v, false, false);
    return (int)((__lane_id() & 32) ? r[0] : r[1]);
  } else if constexpr (MASK > 32) {
    return lane_xor_i32<32>(lane_xor_i32<(MASK & 31)>(v));
  } else if constexpr (MASK > 16) {
    return lane_xor_i32<16>(lane_xor_i32<(MASK & 15)>(v));
  } else {
    return __builtin_amdgcn_ds_swizzle(v, (MASK << 10) | 0x1F);  // bit-mask mode: and 0x1F, or 0, xor MASK
  }
}

template <int MASK>
__device__ __forceinline__ double lane_xor(double v) {
  return __hiloint2double(lane_xor_i32<MASK>(__double2hiint(v)), lane_xor_i32<MASK>(__double2loint(v)));
}

template <int MASK>
__device__ __forceinline__ float lane_xor(float v) {
  return __int_as_float(lane_xor_i32<MASK>(__float_as_int(v)));
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
