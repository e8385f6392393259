// Device-side problem description, workspace header and the importance load shared by all kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tsenor.h"

namespace tsenor_dev {

struct WsHeader {
  unsigned int max_bits;  // bit pattern of the largest importance seen (non-negative floats order as uints)
  unsigned int use_prev;  // safeguard verdict: 1 = the caller's previous mask scores higher and is returned
  double tau_eff;
  unsigned long long stats[4];
  double objective[2];    // sum S*importance of the mask found / of the previous mask
};
static_assert(sizeof(WsHeader) <= 256, "header must fit its slot");

struct DevProblem {
  const void* W;
  const void* add;
  const float* col_scale;
  int64_t ld, cols, nblocks, bc;  // bc: blocks per block-row
  int dtype, N, T, transpose;
  int L, strict;
  double tau;
  int tau_mode;
  float add_scale;
  int square;
};

// One fused launch serves up to kMaxBatch matrices that share M and the kernel variant: every kernel gets the
// table by value, finds the matrix its workgroup belongs to from the prefix `first`, and reads that entry.
// A matrix owns whole workgroups, so the choice is uniform over a workgroup.
constexpr int kMaxBatch = 16;

struct BatchEntry {
  DevProblem p;
  int64_t rows;
  WsHeader* hdr;                // workspace slices of this matrix
  unsigned short* order;
  void* rowmask;
  double* block_objective;      // NULL: no objective asked for
  uint8_t* mask;                // outputs of the caller (NULL where optional and not asked for)
  double* plan_out;
  double* tau_eff_out;
  int64_t* stats_out;
  uint8_t* packed_out;
  void* pruned_out;
  double* objective_out;
  const uint8_t* prev_mask;
  int wide_store;               // mask rows can be written with 16-byte stores
  int absmax_vec;               // rows can be read with 16-byte loads by the maximum pre-pass
};

struct Batch {
  int count;
  unsigned int first[kMaxBatch + 1];  // first workgroup of every matrix in the launch at hand
  BatchEntry e[kMaxBatch];
};
static_assert(sizeof(Batch) <= 4096, "the table travels as a kernel argument");

__device__ __forceinline__ int find_problem(const Batch& b, unsigned int workgroup) {
  int k = 0;
  while (k + 1 < b.count && workgroup >= b.first[k + 1]) ++k;
  return k;
}

__device__ __forceinline__ float load_element(const void* base, int dtype, int64_t index) {
  if (dtype == TSENOR_BF16) {
    const unsigned int b = reinterpret_cast<const unsigned short*>(base)[index];
    return __uint_as_float(b << 16);
  }
  return reinterpret_cast<const float*>(base)[index];
}

// x = W + add_scale * add: the value a kept entry carries (Sec. 4; the ALPS D-update of Proposition 1).
// Explicitly rounded operations: no fused multiply-add, so that a host evaluation gives the same bits.
__device__ __forceinline__ float load_value(const DevProblem& p, int64_t r, int64_t c) {
  const float w = load_element(p.W, p.dtype, r * p.ld + c);
  if (!p.add) return w;
  return __fadd_rn(w, __fmul_rn(p.add_scale, load_element(p.add, p.dtype, r * p.ld + c)));
}

// importance of one weight: |x| (times col_scale[j]) (squared), every step one float operation
// (Sec. 4: Wanda-style scores; Proposition 1: (W + V/rho)^2)
__device__ __forceinline__ float load_importance(const DevProblem& p, int64_t r, int64_t c) {
  float a = fabsf(load_value(p, r, c));
  if (p.col_scale) a = __fmul_rn(a, p.col_scale[c]);
  if (p.square) a = __fmul_rn(a, a);
  return a;
}

// multiplier of the importance in the log-kernel K (App. B.1 parameter choice for the relative mode)
__device__ __forceinline__ double tau_eff_of(const DevProblem& p, const WsHeader* hdr) {
  if (p.tau_mode == TSENOR_TAU_ABSOLUTE) return p.tau;
  float mx = __uint_as_float(hdr->max_bits);
  return mx > 0.0f ? 1.0 / (p.tau * (double)mx) : 0.0;
}

}  // namespace tsenor_dev
