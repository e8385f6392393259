// Kernels behind the optional outputs of a call: the objective of Eq. (1) with the safeguard verdict, and the
// outputs derived from the final mask (bit-packed mask, pruned values).  They do not depend on the block size.
#pragma once
#include "problem.hpp"

namespace tsenor_dev {

// Sum of the per-block objectives in a fixed order (thread t adds blocks t, t+1024, ...; then a tree), and
// the safeguard verdict of App. A.1 (Assumption 1): keep the previous mask if it scores strictly higher.
__global__ __launch_bounds__(1024) void objective_kernel(Batch batch) {
  // one workgroup per matrix of the batch
  const double* block_objective = batch.e[blockIdx.x].block_objective;
  if (!block_objective) return;
  const int64_t nblocks = batch.e[blockIdx.x].p.nblocks;
  const bool have_prev = batch.e[blockIdx.x].prev_mask != nullptr;
  WsHeader* hdr = batch.e[blockIdx.x].hdr;
  double* objective_out = batch.e[blockIdx.x].objective_out;
  __shared__ double part[2][1024];
  double a = 0.0, b = 0.0;
  for (int64_t k = threadIdx.x; k < nblocks; k += 1024) {
    a += block_objective[2 * k];
    b += block_objective[2 * k + 1];
  }
  part[0][threadIdx.x] = a;
  part[1][threadIdx.x] = b;
  __syncthreads();
  for (int s = 512; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) {
      part[0][threadIdx.x] += part[0][threadIdx.x + s];
      part[1][threadIdx.x] += part[1][threadIdx.x + s];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const bool use_prev = have_prev && part[1][0] > part[0][0];
    hdr->objective[0] = part[0][0];
    hdr->objective[1] = part[1][0];
    hdr->use_prev = use_prev ? 1u : 0u;
    if (objective_out) {
      objective_out[0] = use_prev ? part[1][0] : part[0][0];
      objective_out[1] = have_prev ? part[1][0] : 0.0;
    }
  }
}

// Outputs derived from the final mask, 8 consecutive weights of a row per thread: the previous mask copied
// over the new one if the safeguard says so, the bit-packed mask, and the pruned values x * S.
__global__ __launch_bounds__(256) void emit_kernel(Batch batch) {
  // blockIdx.z: matrix of the batch; x and y stride over its 8-weight vectors and rows
  const BatchEntry& e = batch.e[blockIdx.z];
  const uint8_t* prev_mask = e.prev_mask;
  uint8_t* packed_out = e.packed_out;
  void* pruned_out = e.pruned_out;
  if (!prev_mask && !packed_out && !pruned_out) return;
  const DevProblem p = e.p;
  const int64_t rows = e.rows;
  uint8_t* mask = e.mask;
  const bool use_prev = prev_mask && e.hdr->use_prev;
  const int64_t per_row = p.cols / 8;
  // a workgroup handles a contiguous band of rows
  const int64_t band = (rows + gridDim.y - 1) / gridDim.y;
  const int64_t r_end = (blockIdx.y + 1) * band < rows ? (blockIdx.y + 1) * band : rows;
  for (int64_t r = blockIdx.y * band; r < r_end; ++r)
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < per_row; v += (int64_t)gridDim.x * blockDim.x) {
      const int64_t c = v * 8;
      unsigned int bits = 0;
      for (int k = 0; k < 8; ++k) {
        uint8_t s = mask[r * p.cols + c + k];
        if (use_prev) {
          s = prev_mask[r * p.cols + c + k];
          mask[r * p.cols + c + k] = s;
        }
        bits |= (unsigned int)(s & 1) << k;
      }
      if (packed_out) packed_out[r * per_row + v] = (uint8_t)bits;
      if (pruned_out) {
        for (int k = 0; k < 8; ++k) {
          const float x = ((bits >> k) & 1) ? load_value(p, r, c + k) : 0.0f;
          if (p.dtype == TSENOR_BF16) {
            // round to nearest even; x is finite
            const unsigned int u = __float_as_uint(x);
            reinterpret_cast<unsigned short*>(pruned_out)[r * p.cols + c + k] =
                (unsigned short)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
          } else {
            reinterpret_cast<float*>(pruned_out)[r * p.cols + c + k] = x;
          }
        }
      }
    }
}

}  // namespace tsenor_dev
