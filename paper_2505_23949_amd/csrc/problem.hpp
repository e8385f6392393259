// Device-side problem description, workspace header and the importance load shared by all kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tsenor.h"

namespace tsenor_dev {

struct WsHeader {
  unsigned int max_bits;  // bit pattern of the largest importance seen (non-negative floats order as uints)
  unsigned int pad;
  double tau_eff;
  unsigned long long stats[4];
};
static_assert(sizeof(WsHeader) <= 256, "header must fit its slot");

struct DevProblem {
  const void* W;
  const float* col_scale;
  int64_t ld, cols, nblocks, bc;  // bc: blocks per block-row
  int dtype, N, T, transpose;
  int L, strict;
  double tau;
  int tau_mode;
};

// importance of one weight: |w| or |w| * col_scale[j] as one float multiply (Sec. 4, Wanda-style scores)
__device__ __forceinline__ float load_importance(const DevProblem& p, int64_t r, int64_t c) {
  float w;
  if (p.dtype == TSENOR_BF16) {
    unsigned int b = reinterpret_cast<const unsigned short*>(p.W)[r * p.ld + c];
    w = __uint_as_float(b << 16);
  } else {
    w = reinterpret_cast<const float*>(p.W)[r * p.ld + c];
  }
  float a = fabsf(w);
  if (p.col_scale) a = a * p.col_scale[c];
  return a;
}

// multiplier of the importance in the log-kernel K (App. B.1 parameter choice for the relative mode)
__device__ __forceinline__ double tau_eff_of(const DevProblem& p, const WsHeader* hdr) {
  if (p.tau_mode == TSENOR_TAU_ABSOLUTE) return p.tau;
  float mx = __uint_as_float(hdr->max_bits);
  return mx > 0.0f ? 1.0 / (p.tau * (double)mx) : 0.0;
}

}  // namespace tsenor_dev
