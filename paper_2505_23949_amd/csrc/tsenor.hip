// Transposable N:M mask finder for MI355X (gfx950): C ABI, host-side launch logic and the small kernels.
//
// One call enqueues, on the caller's stream, for every group of matrices that share a block size and a
// kernel variant (a single matrix is a group of one):
//   1. init_kernel / absmax_kernel      workspace reset; importance maximum of every matrix (relative tau only)
//   2. dykstra_sort_kernel              tile load, all T Dykstra iterations of Algorithm 1 on chip, sort of
//                                       the M*M plan entries of every block; writes the greedy scan order
//                                       (and the plan if asked for)                       [dykstra_sort.hpp]
//   3. greedy_kernel                    Algorithm 2 lines 1-6, one lane per block (greedy_wide_kernel: M lanes
//                                       per block, for small launches; simple_round_kernel: the ablation arm)
//                                                                                         [rounding.hpp]
//   4. finalize_kernel                  Algorithm 2 lines 7-13 (local search), mask write [rounding.hpp]
//   5. objective_kernel, emit_kernel, stats_kernel   optional outputs                     [outputs.hpp]
// Steps 2-4 depend on the block size and are compiled per M (launch.hpp).  Every kernel takes the table of
// the group by value and finds the matrix of a workgroup from a prefix of workgroup counts.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <cmath>
#include <vector>

#include <mutex>

#include "lanes.hpp"
#include "launch.hpp"
#include "outputs.hpp"
#include "problem.hpp"
#include "tsenor.h"
#include "tsenor_profile.h"

namespace {

using namespace tsenor_dev;

// clears the rounding counters of every matrix of the batch (launched only when a caller asks for them)
__global__ void init_kernel(Batch batch) {
  if ((int)threadIdx.x >= batch.count) return;
  WsHeader* hdr = batch.e[threadIdx.x].hdr;
  for (int k = 0; k < 4; ++k) hdr->stats[k] = 0ull;
}

constexpr int kAbsmaxInFlight = 4;  // rows read per thread before any is used
// threads of a workgroup that share a row: the smallest power of two that covers its vectors
__host__ __device__ inline int absmax_threads_per_row(int64_t vectors_per_row, int threads) {
  int tpr = 1;
  while (tpr < vectors_per_row && tpr < threads) tpr <<= 1;
  return tpr;
}

// Largest importance of every matrix of the batch that uses the relative tau (App. B.1 parameter choice).
// blockIdx.z: matrix; x and y stride over its columns and rows.  With absmax_vec every thread reads 8
// consecutive weights of a row with 16-byte loads (needs cols % 8 == 0 and 16-byte aligned rows and column
// scale); otherwise one weight at a time.  A matrix with fewer than 256 such vectors per row shares the
// workgroup between rows.
__global__ __launch_bounds__(256) void absmax_kernel(Batch batch) {
  const BatchEntry& e = batch.e[blockIdx.z];
  const DevProblem p = e.p;
  if (p.tau_mode != TSENOR_TAU_REL_MATRIX_MAX) return;
  const int64_t rows = e.rows;
  float m = 0.0f;
  if (e.absmax_vec) {
    const int64_t vpr = p.cols / 8;  // 8-weight vectors per row
    // a narrow matrix shares the workgroup between rows: tpr threads per row, blockDim.x / tpr rows per pass
    const int tpr = absmax_threads_per_row(vpr, (int)blockDim.x), rpp = (int)blockDim.x / tpr;
    const int tv = (int)threadIdx.x % tpr, tr = (int)threadIdx.x / tpr;
    for (int64_t v = (int64_t)blockIdx.x * tpr + tv; v < vpr; v += (int64_t)gridDim.x * tpr) {
      float c[8] = {1.0f, 1.0f, 1.0f, 1.0f, 1.0f, 1.0f, 1.0f, 1.0f};  // times exactly 1 where there is no scale
      if (p.col_scale) {
        const float4* cs = reinterpret_cast<const float4*>(p.col_scale + v * 8);
        const float4 a = cs[0], b = cs[1];
        c[0] = a.x, c[1] = a.y, c[2] = a.z, c[3] = a.w, c[4] = b.x, c[5] = b.y, c[6] = b.z, c[7] = b.w;
      }
      // a workgroup streams a contiguous band of rows (rows far apart cost a page-table walk per load)
      const int64_t band = (rows + gridDim.y - 1) / gridDim.y;
      const int64_t r_end = (blockIdx.y + 1) * band < rows ? (blockIdx.y + 1) * band : rows;
      for (int64_t r = blockIdx.y * band + (int64_t)tr * kAbsmaxInFlight; r < r_end; r += (int64_t)rpp * kAbsmaxInFlight) {
        if (p.dtype == TSENOR_BF16) {
          uint4 raw[kAbsmaxInFlight];
#pragma unroll
          for (int u = 0; u < kAbsmaxInFlight; ++u) {
            const int64_t ru = r + u < r_end ? r + u : r;
            raw[u] = *reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned short*>(p.W) + ru * p.ld + v * 8);
          }
#pragma unroll
          for (int u = 0; u < kAbsmaxInFlight; ++u) {
            const unsigned int w[4] = {raw[u].x, raw[u].y, raw[u].z, raw[u].w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
              m = fmaxf(m, fabsf(__uint_as_float(w[k] << 16)) * c[2 * k]);
              m = fmaxf(m, fabsf(__uint_as_float(w[k] & 0xFFFF0000u)) * c[2 * k + 1]);
            }
          }
        } else {
          float4 lo[kAbsmaxInFlight], hi[kAbsmaxInFlight];
#pragma unroll
          for (int u = 0; u < kAbsmaxInFlight; ++u) {
            const int64_t ru = r + u < r_end ? r + u : r;
            const float4* src = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(p.W) + ru * p.ld + v * 8);
            lo[u] = src[0];
            hi[u] = src[1];
          }
#pragma unroll
          for (int u = 0; u < kAbsmaxInFlight; ++u) {
            const float w[8] = {lo[u].x, lo[u].y, lo[u].z, lo[u].w, hi[u].x, hi[u].y, hi[u].z, hi[u].w};
#pragma unroll
            for (int k = 0; k < 8; ++k) m = fmaxf(m, fabsf(w[k]) * c[k]);
          }
        }
      }
    }
  } else {
    for (int64_t r = blockIdx.y; r < rows; r += gridDim.y)
      for (int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; c < p.cols; c += (int64_t)gridDim.x * blockDim.x)
        m = fmaxf(m, load_importance(p, r, c));
  }
  // one partial maximum per workgroup (at most ~512 per matrix); whoever needs the maximum reduces them
  __shared__ float wave_max[4];
  for (int s = 1; s < kWave; s <<= 1) m = fmaxf(m, __shfl_xor(m, s, kWave));
  if ((threadIdx.x & (kWave - 1)) == 0) wave_max[threadIdx.x / kWave] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    m = fmaxf(fmaxf(wave_max[0], wave_max[1]), fmaxf(wave_max[2], wave_max[3]));
    e.absmax_partial[blockIdx.y * gridDim.x + blockIdx.x] = m;
  }
}

__global__ void fill_kernel(uint8_t* mask, int64_t total, uint8_t value) {
  for (int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; k < total; k += (int64_t)gridDim.x * blockDim.x)
    mask[k] = value;
}

__global__ void stats_kernel(Batch batch) {
  const int which = threadIdx.x / 4, k = threadIdx.x % 4;
  if (which < batch.count && batch.e[which].stats_out) batch.e[which].stats_out[k] = (int64_t)batch.e[which].hdr->stats[k];
}

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------

// code of the last HIP failure a call of this thread ran into (hipGetLastError() clears the runtime's own copy)
thread_local int g_last_hip_error = 0;
inline int hip_status_of_launches() {
  const hipError_t e = hipGetLastError();
  if (e == hipSuccess) return TSENOR_OK;
  g_last_hip_error = (int)e;
  return TSENOR_ERR_HIP;
}

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct WsLayout {
  size_t header, partials, order, accept, objective, total;
};

// greedy's output: M row bit masks per block, 32-bit words up to M = 32, 64-bit for M = 64
inline size_t rowmask_bytes_per_block(int M) { return (size_t)M * (M > 32 ? 8 : 4); }

WsLayout layout_of(const tsenor_problem& p) {
  WsLayout l;
  const size_t elems = (size_t)p.rows * (size_t)p.cols;
  const size_t nblocks = elems / ((size_t)p.M * p.M);
  l.header = 0;
  l.partials = kAlign;
  l.order = l.partials + align_up(kMaxAbsmaxPartials * sizeof(float));
  l.accept = l.order + align_up(elems * sizeof(unsigned short));
  l.objective = l.accept + align_up(nblocks * rowmask_bytes_per_block(p.M));
  l.total = l.objective + align_up(nblocks * 2 * sizeof(double));  // per-block objectives (new, previous mask)
  return l;
}

int validate(const tsenor_problem* p) {
  if (!p || !p->W || !p->mask) return TSENOR_ERR_NULL;
  if (p->M != 4 && p->M != 8 && p->M != 16 && p->M != 32 && p->M != 64) return TSENOR_ERR_UNSUPPORTED;
  if (p->dtype != TSENOR_F32 && p->dtype != TSENOR_BF16) return TSENOR_ERR_UNSUPPORTED;
  if (p->tau_mode != TSENOR_TAU_ABSOLUTE && p->tau_mode != TSENOR_TAU_REL_MATRIX_MAX) return TSENOR_ERR_UNSUPPORTED;
  if (p->flags & ~(uint32_t)(TSENOR_FLAG_STRICT_PAPER | TSENOR_FLAG_COLS_FIRST | TSENOR_FLAG_FP32_ITERATIONS |
                             TSENOR_FLAG_GREEDY_ONE_LANE | TSENOR_FLAG_GREEDY_M_LANES | TSENOR_FLAG_TILES_LARGE |
                             TSENOR_FLAG_TILES_SMALL | TSENOR_FLAG_SIMPLE_ROUNDING))
    return TSENOR_ERR_UNSUPPORTED;
  if ((p->flags & TSENOR_FLAG_GREEDY_ONE_LANE) && (p->flags & TSENOR_FLAG_GREEDY_M_LANES)) return TSENOR_ERR_PARAM;
  if ((p->flags & TSENOR_FLAG_TILES_LARGE) && (p->flags & TSENOR_FLAG_TILES_SMALL)) return TSENOR_ERR_PARAM;
  if (p->rows <= 0 || p->cols <= 0 || p->rows % p->M || p->cols % p->M || p->ld < p->cols) return TSENOR_ERR_SHAPE;
  if (p->rows > (int64_t)1 << 31 || p->cols > (int64_t)1 << 31 || p->rows * p->cols > (int64_t)1 << 40)
    return TSENOR_ERR_SHAPE;
  if (p->N < 0 || p->N > p->M) return TSENOR_ERR_NM;
  if (!(p->tau > 0.0) || !std::isfinite(p->tau) || p->iters < 0 || p->local_search_steps < 0) return TSENOR_ERR_PARAM;
  if (p->tau_mode == TSENOR_TAU_REL_MATRIX_MAX && p->tau < 1.0 / 690.0) return TSENOR_ERR_PARAM;
  if (p->importance != TSENOR_IMPORTANCE_ABS && p->importance != TSENOR_IMPORTANCE_SQUARE) return TSENOR_ERR_UNSUPPORTED;
  if (p->add && !std::isfinite(p->add_scale)) return TSENOR_ERR_PARAM;
  if ((p->packed_out || p->pruned_out || p->prev_mask) && p->cols % 8) return TSENOR_ERR_SHAPE;
  if ((p->N == 0 || p->N == p->M) && (p->objective_out || p->prev_mask || p->iters_done_out)) return TSENOR_ERR_UNSUPPORTED;
  if (!(p->tol >= 0.0) || !std::isfinite(p->tol)) return TSENOR_ERR_PARAM;
  return TSENOR_OK;
}

inline bool degenerate(const tsenor_problem& p) { return p.N == 0 || p.N == p.M; }

inline Variant variant_of(const tsenor_problem& p) {
  Variant v;
  v.M = p.M;
  v.zero_t = p.iters == 0;
  v.greedy = p.flags & (uint32_t)(TSENOR_FLAG_GREEDY_ONE_LANE | TSENOR_FLAG_GREEDY_M_LANES);
  v.simple = (p.flags & TSENOR_FLAG_SIMPLE_ROUNDING) != 0;
  // the tiling is decided from the matrix's own number of blocks, never from what it is fused with: the two
  // tilings differ in the order of the additions inside a row or column sum
  const int64_t nblocks = (p.rows / p.M) * (p.cols / p.M);
  const bool fp32 = (p.flags & TSENOR_FLAG_FP32_ITERATIONS) != 0;
  v.small = p.M <= 32 && !v.zero_t && !v.simple &&
            ((p.flags & TSENOR_FLAG_TILES_SMALL) != 0 ||
             (!(p.flags & TSENOR_FLAG_TILES_LARGE) && nblocks < small_tiles_below_blocks(p.M, fp32)));
  // the small tiles (launches that cannot fill the chip: bound by latency, not by issue) iterate in double only
  v.fast = p.iters > 0 && fp32 && !v.small;
  v.adaptive = p.tol > 0.0 && p.iters > 0;
  return v;
}

BatchEntry entry_of(const tsenor_problem& p, char* ws) {
  const WsLayout l = layout_of(p);
  BatchEntry e = {};
  DevProblem& dp = e.p;
  dp.W = p.W;
  dp.add = p.add;
  dp.add_scale = p.add ? p.add_scale : 0.0f;
  dp.square = p.importance == TSENOR_IMPORTANCE_SQUARE;
  dp.col_scale = p.col_scale;
  dp.ld = p.ld;
  dp.cols = p.cols;
  dp.bc = p.cols / p.M;
  dp.nblocks = (p.rows / p.M) * dp.bc;
  dp.dtype = p.dtype;
  dp.N = p.N;
  dp.T = p.iters;
  dp.transpose = (p.flags & TSENOR_FLAG_COLS_FIRST) ? 1 : 0;
  dp.L = p.local_search_steps;
  dp.strict = (p.flags & TSENOR_FLAG_STRICT_PAPER) ? 1 : 0;
  if (p.flags & TSENOR_FLAG_SIMPLE_ROUNDING) {
    dp.L = 0;  // the simple arm has no local search: the last kernel only writes the mask
    dp.strict = 1;
  }
  dp.tau = p.tau;
  dp.tau_mode = p.tau_mode;
  dp.tol = p.tol;
  e.rows = p.rows;
  e.hdr = reinterpret_cast<WsHeader*>(ws + l.header);
  e.absmax_partial = reinterpret_cast<float*>(ws + l.partials);
  e.absmax_count = 0;  // set with the grid of the pre-pass
  e.order = reinterpret_cast<unsigned short*>(ws + l.order);
  e.rowmask = ws + l.accept;
  e.block_objective = (p.objective_out || p.prev_mask) ? reinterpret_cast<double*>(ws + l.objective) : nullptr;
  e.mask = p.mask;
  e.plan_out = p.plan_out;
  e.tau_eff_out = p.tau_eff_out;
  e.stats_out = p.stats_out;
  e.packed_out = p.packed_out;
  e.pruned_out = p.pruned_out;
  e.objective_out = p.objective_out;
  e.prev_mask = p.prev_mask;
  e.iters_done_out = p.iters_done_out;
  e.wide_store = reinterpret_cast<uintptr_t>(p.mask) % 16 == 0;
  const size_t esize = p.dtype == TSENOR_BF16 ? 2 : 4;
  e.absmax_vec = p.cols % 8 == 0 && reinterpret_cast<uintptr_t>(p.W) % 16 == 0 && ((size_t)p.ld * esize) % 16 == 0 &&
                 reinterpret_cast<uintptr_t>(p.col_scale) % 16 == 0 && !p.add && !dp.square;
  return e;
}

// grid of the kernels that stride over a matrix 8 weights (or 1) at a time: x over a row, y over rows,
// about `target` workgroups in all, sized for the largest matrix of the batch
dim3 strided_grid(const Batch& b, bool vec_only, unsigned target, bool for_absmax) {
  unsigned gx = 1, gy = 1;
  for (int k = 0; k < b.count; ++k) {
    const BatchEntry& e = b.e[k];
    const int64_t per_row = (vec_only || e.absmax_vec) ? e.p.cols / 8 : e.p.cols;
    const unsigned x = (unsigned)std::min<int64_t>((per_row + 255) / 256, 16);
    gx = std::max(gx, x);
    int64_t bands = std::min<int64_t>(e.rows, std::max<unsigned>(target / x, 1));
    if (for_absmax && e.absmax_vec) {
      // enough rows per workgroup to give every thread its rows in flight (a narrow matrix shares the
      // workgroup between rows), and no more workgroups than that: each leaves a partial maximum to be reduced
      const int64_t rows_per_group = (int64_t)(256 / absmax_threads_per_row(per_row, 256)) * kAbsmaxInFlight;
      bands = std::min(bands, (e.rows + rows_per_group - 1) / rows_per_group);
    }
    gy = std::max(gy, (unsigned)bands);
  }
  // (matrices of different shapes can ask for a wide and for a tall grid: the product stays within the
  // partial maxima a workspace holds; the kernels stride by the grid they get)
  if (for_absmax) gy = std::min(gy, (unsigned)kMaxAbsmaxPartials / gx);
  return dim3(gx, gy, (unsigned)b.count);
}

// A fused launch gives every block at least a lane and at most a workgroup of its own, so its grids hold as
// long as the blocks of the group number fewer than 2^31.
constexpr int64_t kMaxBlocksPerLaunch = 0x7FFFFFFF;

// All kernels of one fused launch: `b.count` non-degenerate problems of the same variant.
// ev (optional): TSENOR_NUM_STAGES + 1 events recorded at the stage boundaries.
int run_group(Batch& b, const Variant& v, hipStream_t stream, hipEvent_t* ev = nullptr) {
  auto mark = [&](int k) {
    if (ev) (void)hipEventRecord(ev[k], stream);
  };
  bool any_rel = false, any_objective = false, any_emit = false, any_stats = false;
  for (int k = 0; k < b.count; ++k) {
    const BatchEntry& e = b.e[k];
    any_rel |= e.p.tau_mode == TSENOR_TAU_REL_MATRIX_MAX;
    any_objective |= e.block_objective != nullptr;
    any_emit |= e.packed_out || e.pruned_out || e.prev_mask;
    any_stats |= e.stats_out != nullptr;
  }
  mark(0);
  if (any_stats) init_kernel<<<1, kMaxBatch, 0, stream>>>(b);
  if (any_rel) {
    const dim3 grid = strided_grid(b, false, 512, true);
    for (int k = 0; k < b.count; ++k) b.e[k].absmax_count = (int)(grid.x * grid.y);
    absmax_kernel<<<grid, 256, 0, stream>>>(b);
  }
  mark(1);
  hipEvent_t ev_sorted = ev ? ev[2] : nullptr, ev_greedy = ev ? ev[3] : nullptr;
  bool ok = false;
  switch (v.M) {
    case 4: ok = launch_block_kernels<4>(b, v, stream, ev_sorted, ev_greedy); break;
    case 8: ok = launch_block_kernels<8>(b, v, stream, ev_sorted, ev_greedy); break;
    case 16: ok = launch_block_kernels<16>(b, v, stream, ev_sorted, ev_greedy); break;
    case 32: ok = launch_block_kernels<32>(b, v, stream, ev_sorted, ev_greedy); break;
    case 64: ok = launch_block_kernels<64>(b, v, stream, ev_sorted, ev_greedy); break;
  }
  if (!ok) return TSENOR_ERR_SHAPE;  // (ruled out by the checks before the first launch)
  if (any_objective) objective_kernel<<<b.count, 1024, 0, stream>>>(b);
  if (any_emit) emit_kernel<<<strided_grid(b, true, 2048, false), 256, 0, stream>>>(b);
  if (any_stats) stats_kernel<<<1, 4 * kMaxBatch, 0, stream>>>(b);
  mark(4);
  return hip_status_of_launches();
}

// N = 0 and N = M need no solve: the mask is constant and the statistics are zero.
int run_degenerate(const tsenor_problem& p, char* ws, hipStream_t stream, hipEvent_t* ev = nullptr) {
  const int64_t total = p.rows * p.cols;
  const int grid = (int)std::min<int64_t>((total + 255) / 256, 65535);
  if (ev)
    for (int k = 0; k < 4; ++k) (void)hipEventRecord(ev[k], stream);
  fill_kernel<<<grid, 256, 0, stream>>>(p.mask, total, p.N == 0 ? 0 : 1);
  Batch b = {};
  b.count = 1;
  b.e[0] = entry_of(p, ws);
  if (p.stats_out) {
    init_kernel<<<1, kMaxBatch, 0, stream>>>(b);
    stats_kernel<<<1, 4 * kMaxBatch, 0, stream>>>(b);
  }
  if (p.packed_out || p.pruned_out) emit_kernel<<<strided_grid(b, true, 2048, false), 256, 0, stream>>>(b);
  if (ev) (void)hipEventRecord(ev[4], stream);
  return hip_status_of_launches();
}

// Everything a call checks before it enqueues anything: every problem on its own, the workspace, and that the
// fused launches can be described.  `need` receives the workspace bytes of the call.
int check_call(const tsenor_problem* problems, int count, const void* workspace, size_t workspace_bytes) {
  if (!problems || count <= 0) return TSENOR_ERR_NULL;
  size_t need = 0;
  for (int k = 0; k < count; ++k) {
    const int rc = validate(&problems[k]);
    if (rc != TSENOR_OK) return rc;
    need += layout_of(problems[k]).total;
  }
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % kAlign) || workspace_bytes < need)
    return TSENOR_ERR_WORKSPACE;
  // blocks per block size: an upper bound of what any fused launch of the call holds
  int64_t blocks_of_m[65] = {};
  for (int k = 0; k < count; ++k) {
    const tsenor_problem& p = problems[k];
    if (degenerate(p)) continue;
    blocks_of_m[p.M] += (p.rows / p.M) * (p.cols / p.M);
    if (blocks_of_m[p.M] > kMaxBlocksPerLaunch) return TSENOR_ERR_SHAPE;
  }
  return TSENOR_OK;
}

// One checked problem (no host allocation on this path).  Only a failing HIP call can stop it.
int run_one(const tsenor_problem& p, char* ws, hipStream_t s, hipEvent_t* ev = nullptr) {
  if (degenerate(p)) return run_degenerate(p, ws, s, ev);
  Batch b = {};
  b.count = 1;
  b.e[0] = entry_of(p, ws);
  return run_group(b, variant_of(p), s, ev);
}

// The checked problems of a batch, group by group.  Only a failing HIP call can stop this once it has started.
int run_checked(const tsenor_problem* problems, int count, char* base, hipStream_t s) {
  if (count == 1) return run_one(problems[0], base, s);
  // workspace slice of every problem, in the order given
  std::vector<size_t> offset((size_t)count);
  size_t at = 0;
  for (int k = 0; k < count; ++k) {
    offset[(size_t)k] = at;
    at += layout_of(problems[k]).total;
  }
  // problems that run the same kernel variant share fused launches, up to kMaxBatch matrices each
  std::vector<char> done((size_t)count, 0);
  for (int k = 0; k < count; ++k) {
    if (done[(size_t)k]) continue;
    if (degenerate(problems[k])) {
      const int rc = run_degenerate(problems[k], base + offset[(size_t)k], s);
      if (rc != TSENOR_OK) return rc;
      done[(size_t)k] = 1;
      continue;
    }
    const Variant v = variant_of(problems[k]);
    Batch b = {};
    for (int j = k; j < count && b.count < kMaxBatch; ++j) {
      if (done[(size_t)j] || degenerate(problems[j]) || !(variant_of(problems[j]) == v)) continue;
      b.e[b.count++] = entry_of(problems[j], base + offset[(size_t)j]);
      done[(size_t)j] = 1;
    }
    const int rc = run_group(b, v, s);
    if (rc != TSENOR_OK) return rc;
  }
  return TSENOR_OK;
}

// ------------------------------------------------------------------------------------------------
// Scratch of tsenor_mask_ex_static: a fixed array in device memory, one copy per GPU, held from the moment the
// library's code is loaded on that GPU until the process ends.  Host code never uses the array's name as an
// address: the device address is looked up once per device and kept.
// ------------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[TSENOR_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
void* g_scratch_ptr[kMaxDevices] = {};

// device address of `scratch` on the current device (nullptr on failure)
void* static_scratch_of_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> hold(g_scratch_lock);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

}  // namespace

extern "C" {

size_t tsenor_workspace_bytes(const tsenor_problem* problems, int count) {
  if (!problems || count <= 0) return 0;
  size_t total = 0;
  for (int k = 0; k < count; ++k) {
    if (validate(&problems[k]) != TSENOR_OK) return 0;
    total += layout_of(problems[k]).total;
  }
  return total;
}

int tsenor_mask_batched(const tsenor_problem* problems, int count, void* workspace, size_t workspace_bytes,
                        tsenor_stream_t stream) {
  const int rc = check_call(problems, count, workspace, workspace_bytes);
  if (rc != TSENOR_OK) return rc;
  return run_checked(problems, count, static_cast<char*>(workspace), static_cast<hipStream_t>(stream));
}

int tsenor_mask_ex(const tsenor_problem* p, void* workspace, size_t workspace_bytes, tsenor_stream_t stream) {
  return tsenor_mask_batched(p, 1, workspace, workspace_bytes, stream);
}

int tsenor_mask_ex_static(const tsenor_problem* p, tsenor_stream_t stream) {
  if (!p) return TSENOR_ERR_NULL;
  const int rc = validate(p);
  if (rc != TSENOR_OK) return rc;
  if (layout_of(*p).total > (size_t)TSENOR_STATIC_SCRATCH_BYTES) return TSENOR_ERR_TOO_LARGE;
  void* ptr = static_scratch_of_current_device();
  if (!ptr) return TSENOR_ERR_HIP;
  const int rc2 = check_call(p, 1, ptr, (size_t)TSENOR_STATIC_SCRATCH_BYTES);
  if (rc2 != TSENOR_OK) return rc2;
  return run_one(*p, static_cast<char*>(ptr), static_cast<hipStream_t>(stream));
}

int tsenor_mask_ex_profile(const tsenor_problem* p, void* workspace, size_t workspace_bytes, tsenor_stream_t stream,
                           int repeats, float* stage_ms, double* loop_clock_mhz) {
  if (!p || !stage_ms) return TSENOR_ERR_NULL;
  const int rc = check_call(p, 1, workspace, workspace_bytes);
  if (rc != TSENOR_OK) return rc;
  if (repeats <= 0 || repeats > 4096) return TSENOR_ERR_PARAM;
  hipStream_t s = static_cast<hipStream_t>(stream);
  constexpr int NE = TSENOR_NUM_STAGES + 1;
  hipEvent_t* ev = new hipEvent_t[(size_t)repeats * NE];
  int created = 0, out = TSENOR_OK;
  for (; created < repeats * NE; ++created)
    if (hipEventCreate(&ev[created]) != hipSuccess) {
      out = TSENOR_ERR_HIP;
      break;
    }
  for (int r = 0; r < repeats && out == TSENOR_OK; ++r)
    out = run_one(*p, static_cast<char*>(workspace), s, ev + r * NE);
  if (out == TSENOR_OK && hipStreamSynchronize(s) != hipSuccess) out = TSENOR_ERR_HIP;
  for (int k = 0; k < TSENOR_NUM_STAGES; ++k) stage_ms[k] = 0.0f;
  for (int r = 0; r < repeats && out == TSENOR_OK; ++r)
    for (int k = 0; k < TSENOR_NUM_STAGES; ++k) {
      float ms = 0.0f;
      if (hipEventElapsedTime(&ms, ev[r * NE + k], ev[r * NE + k + 1]) != hipSuccess) out = TSENOR_ERR_HIP;
      stage_ms[k] += ms / (float)repeats;
    }
  for (int k = 0; k < created; ++k) (void)hipEventDestroy(ev[k]);
  delete[] ev;
  if (loop_clock_mhz) {
    *loop_clock_mhz = 0.0;
    WsHeader h;
    int dev = 0, khz = 0;
    if (out == TSENOR_OK && !degenerate(*p) && p->iters > 0 &&
        hipMemcpy(&h, workspace, sizeof(h), hipMemcpyDeviceToHost) == hipSuccess && h.loop_ticks > 0 &&
        hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) == hipSuccess)
      *loop_clock_mhz = (double)h.loop_cycles / (double)h.loop_ticks * (double)khz * 1e-3;
  }
  return out;
}

int tsenor_mask(const float* W, int64_t rows, int64_t cols, int N, int M, float tau, int iters, uint8_t* mask,
                tsenor_stream_t stream) {
  tsenor_problem p = {};
  p.W = W;
  p.dtype = TSENOR_F32;
  p.rows = rows;
  p.cols = cols;
  p.ld = cols;
  p.N = N;
  p.M = M;
  p.tau = (double)tau;
  p.tau_mode = TSENOR_TAU_ABSOLUTE;
  p.iters = iters;
  p.local_search_steps = 10;
  p.mask = mask;
  const int rc = validate(&p);
  if (rc != TSENOR_OK) return rc;
  const size_t bytes = layout_of(p).total;
  void* ws = nullptr;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (hipMallocAsync(&ws, bytes, s) != hipSuccess) return TSENOR_ERR_HIP;
  const int rc2 = tsenor_mask_batched(&p, 1, ws, bytes, stream);
  if (hipFreeAsync(ws, s) != hipSuccess) return TSENOR_ERR_HIP;
  return rc2;
}

const char* tsenor_status_string(int status) {
  switch (status) {
    case TSENOR_OK: return "ok";
    case TSENOR_ERR_NULL: return "a required pointer is NULL";
    case TSENOR_ERR_SHAPE: return "rows/cols must be positive multiples of M, ld >= cols, at most 2^40 weights and fewer than 2^31 blocks of one size per call";
    case TSENOR_ERR_NM: return "N must satisfy 0 <= N <= M";
    case TSENOR_ERR_UNSUPPORTED: return "unsupported M (4, 8, 16, 32, 64), dtype, tau_mode or flag";
    case TSENOR_ERR_PARAM: return "tau must be finite and > 0 (>= 1/690 in REL_MATRIX_MAX mode), iters and local_search_steps >= 0, at most one TSENOR_FLAG_GREEDY_* and one TSENOR_FLAG_TILES_* flag";
    case TSENOR_ERR_WORKSPACE: return "workspace is NULL, not 256-byte aligned or smaller than tsenor_workspace_bytes";
    case TSENOR_ERR_HIP: return "a HIP call failed";
    case TSENOR_ERR_TOO_LARGE: return "tsenor_mask_ex_static: the problem needs more scratch than TSENOR_STATIC_SCRATCH_BYTES; use tsenor_mask_ex with a workspace";
  }
  return "unknown status";
}

int tsenor_last_hip_error(void) { return g_last_hip_error; }

int tsenor_version(void) { return 200; }

}  // extern "C"
