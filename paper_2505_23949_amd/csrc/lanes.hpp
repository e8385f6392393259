// Cross-lane data movement for 64-wide wavefronts on gfx950.
//
// lane_xor<MASK>(v) returns v of lane (lane ^ MASK).  Mechanism per mask, chosen by measurement on MI355X
// (the kernels that use this are bound by vector-ALU issue):
//   1, 2, 3   DPP quad_perm          7   DPP row_half_mirror      15  DPP row_mirror      8  DPP row_ror:8
//             one v_mov_b32_dpp per 32 bits (the compiler folds it into a 32-bit add/mul where it can);
//   other masks below 32: ds_swizzle in bit-mask mode (LDS crossbar, no LDS memory).  It issues on the LDS
//             pipeline, so it costs no vector-ALU slot; its ~100 cycles of latency are hidden by the second
//             wave of the SIMD.  For xor 16 this beat v_permlane16_swap + select by 4 %, for xor 4 it beat
//             two bank-masked DPP row shifts by 5 %; routing the DPP-able masks through it as well was 3 %
//             slower (the latency then shows).
//   32        v_permlane32_swap + select; masks above 32: xor 32 composed with the rest.
// ds_bpermute-based shuffles (__shfl_xor) cost about four times a DPP move per 64-bit value and are not used.
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
  } else if constexpr (MASK < 32) {
    return __builtin_amdgcn_ds_swizzle(v, (MASK << 10) | 0x1F);  // bit-mask mode: and 0x1F, or 0, xor MASK
  } else if constexpr (MASK == 32) {
    // swaps lanes 32..63 of the first operand with lanes 0..31 of the second
    const auto r = __builtin_amdgcn_permlane32_swap((unsigned)v, (unsigned)v, false, false);
    return (int)((__lane_id() & 32) ? r[0] : r[1]);
  } else {
    return lane_xor_i32<32>(lane_xor_i32<(MASK & 31)>(v));
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

// max over the LPB consecutive lanes that hold a block (LPB a power of two)
template <int LPB, int STEP = 1>
__device__ __forceinline__ double block_max(double v) {
  if constexpr (STEP < LPB) {
    v = fmax(v, lane_xor<STEP>(v));
    return block_max<LPB, STEP * 2>(v);
  } else {
    return v;
  }
}

}  // namespace tsenor_dev
