// Device-side problem description, workspace header and the importance load shared by all kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tsenor.h"

namespace tsenor_dev {

// Head of a matrix's workspace slice: what the kernels of a call pass to each other besides the scan order.
struct WsHeader {
  unsigned int use_prev;  // safeguard verdict: 1 = the caller's previous mask scores higher and is returned
  unsigned long long stats[4];  // the four rounding counters (accumulated only when the caller asks for them)
  double objective[2];    // sum S*importance of the mask found / of the previous mask
  // measurement aid: shader-clock cycles and constant-rate timer ticks that the first wave of the Dykstra kernel
  // spent in its iteration loop (their ratio is the clock the chip held under that load)
  unsigned long long loop_cycles, loop_ticks;
};
static_assert(sizeof(WsHeader) <= 256, "header must fit its slot");

// The importance maximum of a matrix (relative tau) travels as one partial maximum per workgroup of the
// pre-pass, in the workspace right after the header; the kernel that needs the maximum reduces them itself.
// No atomic, so nothing has to be cleared before a call.
constexpr int kMaxAbsmaxPartials = 1024;

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
  double tol;  // > 0: early exit of the iterations (see tsenor_problem.tol)
};

// One fused launch serves up to kMaxBatch matrices that share M and the kernel variant: every kernel gets the
// table by value, finds the matrix its workgroup belongs to from the prefix `first`, and reads that entry.
// A matrix owns whole workgroups, so the choice is uniform over a workgroup.
constexpr int kMaxBatch = 16;

struct BatchEntry {
  DevProblem p;
  int64_t rows;
  WsHeader* hdr;                // workspace slices of this matrix
  float* absmax_partial;        // partial maxima of the importance, absmax_count of them (relative tau only)
  int absmax_count;
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
  int* iters_done_out;
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

// Tile loads.  A lane holds a TH x TW register tile of its block; the element offset of tile entry (a, b)
// is base + roff[a] + coff[b], and its column scale is csa[a] * csb[b] where one of the two factors is
// exactly 1 (which of them depends on whether the kernel works on the block or on its transpose), so the
// product with both is still the single rounded multiply of the definition above.  The point of this form:
// every choice (storage type, additive term, scale, transpose) is made once per tile, and the loads of a
// tile are one straight run of independent instructions instead of a chain of branches with a wait each.
template <int TH, int TW>
struct TileAddr {
  int64_t base;
  int64_t roff[TH], coff[TW];
  float csa[TH], csb[TW];
};

// ri[a], cj[b]: coordinates of the tile's rows and columns inside the (possibly transposed) block at
// matrix position (r0, c0)
template <int TH, int TW>
__device__ __forceinline__ TileAddr<TH, TW> tile_addr(const DevProblem& p, int64_t r0, int64_t c0, const int (&ri)[TH],
                                                      const int (&cj)[TW]) {
  TileAddr<TH, TW> t;
  t.base = r0 * p.ld + c0;
#pragma unroll
  for (int a = 0; a < TH; ++a) {
    t.roff[a] = p.transpose ? (int64_t)ri[a] : ri[a] * p.ld;
    t.csa[a] = 1.0f;
  }
#pragma unroll
  for (int b = 0; b < TW; ++b) {
    t.coff[b] = p.transpose ? cj[b] * p.ld : (int64_t)cj[b];
    t.csb[b] = 1.0f;
  }
  if (p.col_scale) {
    if (p.transpose) {
#pragma unroll
      for (int a = 0; a < TH; ++a) t.csa[a] = p.col_scale[c0 + ri[a]];
    } else {
#pragma unroll
      for (int b = 0; b < TW; ++b) t.csb[b] = p.col_scale[c0 + cj[b]];
    }
  }
  return t;
}

template <bool BF16, bool ADD, int A0, int NA, int TH, int TW>
__device__ __forceinline__ void tile_values(const DevProblem& p, const TileAddr<TH, TW>& t, float (&x)[NA][TW]) {
  float v[ADD ? NA : 1][ADD ? TW : 1];
#pragma unroll
  for (int a = 0; a < NA; ++a)
#pragma unroll
    for (int b = 0; b < TW; ++b) {
      const int64_t off = t.base + t.roff[A0 + a] + t.coff[b];
      if constexpr (BF16) {
        x[a][b] = __uint_as_float((unsigned int)reinterpret_cast<const unsigned short*>(p.W)[off] << 16);
        if constexpr (ADD) v[a][b] = __uint_as_float((unsigned int)reinterpret_cast<const unsigned short*>(p.add)[off] << 16);
      } else {
        x[a][b] = reinterpret_cast<const float*>(p.W)[off];
        if constexpr (ADD) v[a][b] = reinterpret_cast<const float*>(p.add)[off];
      }
    }
  if constexpr (ADD) {
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
      for (int b = 0; b < TW; ++b) x[a][b] = __fadd_rn(x[a][b], __fmul_rn(p.add_scale, v[a][b]));
  }
}

// importance of tile rows [A0, A0 + NA): the same operations, in the same order, as load_importance
template <int A0, int NA, int TH, int TW>
__device__ __forceinline__ void tile_importance(const DevProblem& p, const TileAddr<TH, TW>& t, float (&imp)[NA][TW]) {
  if (p.dtype == TSENOR_BF16) {
    if (p.add)
      tile_values<true, true, A0, NA>(p, t, imp);
    else
      tile_values<true, false, A0, NA>(p, t, imp);
  } else {
    if (p.add)
      tile_values<false, true, A0, NA>(p, t, imp);
    else
      tile_values<false, false, A0, NA>(p, t, imp);
  }
#pragma unroll
  for (int a = 0; a < NA; ++a)
#pragma unroll
    for (int b = 0; b < TW; ++b) {
      float m = __fmul_rn(__fmul_rn(fabsf(imp[a][b]), t.csa[A0 + a]), t.csb[b]);
      if (p.square) m = __fmul_rn(m, m);
      imp[a][b] = m;
    }
}

// importance of the M entries (r0 .. r0+M-1, c) of one matrix column, loads issued together; the same
// operations, in the same order, as load_importance
template <int M, bool BF16, bool ADD>
__device__ __forceinline__ void block_column_values(const DevProblem& p, int64_t r0, int64_t c, float (&x)[M]) {
  float v[ADD ? M : 1];
#pragma unroll
  for (int k = 0; k < M; ++k) {
    const int64_t off = (r0 + k) * p.ld + c;
    if constexpr (BF16) {
      x[k] = __uint_as_float((unsigned int)reinterpret_cast<const unsigned short*>(p.W)[off] << 16);
      if constexpr (ADD) v[k] = __uint_as_float((unsigned int)reinterpret_cast<const unsigned short*>(p.add)[off] << 16);
    } else {
      x[k] = reinterpret_cast<const float*>(p.W)[off];
      if constexpr (ADD) v[k] = reinterpret_cast<const float*>(p.add)[off];
    }
  }
  if constexpr (ADD) {
#pragma unroll
    for (int k = 0; k < M; ++k) x[k] = __fadd_rn(x[k], __fmul_rn(p.add_scale, v[k]));
  }
}
template <int M>
__device__ __forceinline__ void block_column_importance(const DevProblem& p, int64_t r0, int64_t c, float (&imp)[M]) {
  if (p.dtype == TSENOR_BF16) {
    if (p.add)
      block_column_values<M, true, true>(p, r0, c, imp);
    else
      block_column_values<M, true, false>(p, r0, c, imp);
  } else {
    if (p.add)
      block_column_values<M, false, true>(p, r0, c, imp);
    else
      block_column_values<M, false, false>(p, r0, c, imp);
  }
  const float cs = p.col_scale ? p.col_scale[c] : 1.0f;
#pragma unroll
  for (int k = 0; k < M; ++k) {
    float m = __fmul_rn(fabsf(imp[k]), cs);  // times exactly 1 where there is no scale
    if (p.square) m = __fmul_rn(m, m);
    imp[k] = m;
  }
}

// multiplier of the importance in the log-kernel K (App. B.1 parameter choice for the relative mode).
// Called by whole waves: the partial maxima of the pre-pass are reduced across the lanes.
__device__ __forceinline__ double tau_eff_of(const BatchEntry& e) {
  const DevProblem& p = e.p;
  if (p.tau_mode == TSENOR_TAU_ABSOLUTE) return p.tau;
  float mx = 0.0f;
  for (int k = (int)(threadIdx.x & 63u); k < e.absmax_count; k += 64) mx = fmaxf(mx, e.absmax_partial[k]);
  for (int s = 1; s < 64; s <<= 1) mx = fmaxf(mx, __shfl_xor(mx, s, 64));
  return mx > 0.0f ? 1.0 / (p.tau * (double)mx) : 0.0;
}

}  // namespace tsenor_dev
