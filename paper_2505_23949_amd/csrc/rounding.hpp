// Algorithm 2: greedy selection (one lane per block) and local search plus the mask write.
#pragma once
#include <limits>
#include <type_traits>

#include "lanes.hpp"
#include "problem.hpp"

namespace tsenor_dev {

// Bit masks over the M columns (or rows) of a block.
template <int M>
using block_mask_t = typename std::conditional<(M > 32), unsigned long long, unsigned int>::type;

template <class mask_t>
__device__ __forceinline__ int mask_popc(mask_t v) {
  if constexpr (sizeof(mask_t) == 8)
    return __popcll((unsigned long long)v);
  else
    return __popc((unsigned int)v);
}

// Waves per workgroup of greedy_kernel.  A full matrix gives the kernel about one wave per SIMD (57 344 blocks: 896
// waves for 1024 SIMDs), and a wave's pace is its own dependent chain: it must not share a SIMD while others
// idle.  One-wave workgroups were placed unevenly (0.096 ms for the headline matrix); workgroups of four waves, one
// per SIMD of a CU, take 0.077 ms.  (M = 64 keeps one wave: its 36 KB of LDS per wave already spread the
// workgroups, and four waves measured the same.)  The waves of a workgroup do not interact.
template <int M>
constexpr int kGreedyWaves = M <= 32 ? 4 : 1;

// Algorithm 2 lines 1-6: scan the entries of a block in sorted order and keep an entry while its row
// and its column hold fewer than N.  The chain of M*M dependent steps runs with ONE LANE PER BLOCK, so
// every lane of the wave does useful work; the state of a lane (M row masks, M column counters) lives in
// LDS.  The kernel is bound by the instruction issue of its single wave per SIMD (~27 instructions per
// entry), not by memory: the scan order is prefetched a cache line ahead and the LDS state of four entries
// is fetched per round trip.  Output: the mask as M row bit masks per block (bit c of word r = S[r][c]).
template <int M>
__global__ __launch_bounds__(kWave * kGreedyWaves<M>) void greedy_kernel(Batch batch) {
  using mask_t = block_mask_t<M>;
  constexpr int MM = M * M;
  __shared__ mask_t rowbits_[kGreedyWaves<M>][M][kWave];
  __shared__ unsigned char colcnt_[kGreedyWaves<M>][M][kWave];
  auto& rowbits = rowbits_[threadIdx.x / kWave];
  auto& colcnt = colcnt_[threadIdx.x / kWave];
  // `vgroup` counts 64-block groups across the launch, as the group prefix of the batch does
  const unsigned int vgroup = blockIdx.x * kGreedyWaves<M> + threadIdx.x / kWave;
  if (vgroup >= batch.first[batch.count]) return;  // (a whole wave; the kernel has no barrier)
  const int which = find_problem(batch, vgroup);
  const unsigned short* order = batch.e[which].order;
  const int64_t nblocks = batch.e[which].p.nblocks;
  const int N = batch.e[which].p.N;
  mask_t* rowmask = static_cast<mask_t*>(batch.e[which].rowmask);
  WsHeader* hdr = batch.e[which].hdr;
  const int lane = threadIdx.x % kWave;
  const int64_t blk = (int64_t)(vgroup - batch.first[which]) * kWave + lane;
  for (int k = 0; k < M; ++k) {
    rowbits[k][lane] = 0;
    colcnt[k][lane] = 0;
  }
  int missing = 0;
  if (blk < nblocks) {
    const unsigned short* src = order + blk * MM;
    int placed = 0;
    const int need = N * M;
    // the scan order arrives 8 entries per 16-byte load; the D loads of the next 8*D entries (one 128-byte
    // line of this lane's block for D = 8) are in flight while the current 8*D entries are decided
    constexpr int D = MM / 8 < 8 ? MM / 8 : 8;
    uint4 cur[D], nxt[D];
#pragma unroll
    for (int d = 0; d < D; ++d) nxt[d] = cur[d] = *reinterpret_cast<const uint4*>(src + 8 * d);
    for (int h0 = 0; h0 < MM && placed < need; h0 += 8 * D) {
      if (h0 + 8 * D < MM) {
#pragma unroll
        for (int d = 0; d < D; ++d) nxt[d] = *reinterpret_cast<const uint4*>(src + h0 + 8 * D + 8 * d);
      }
#pragma unroll
      for (int d = 0; d < D; ++d) {
      const uint4 v = cur[d];
      const unsigned int pk[4] = {v.x, v.y, v.z, v.w};
      // four entries per step: their rows' masks and columns' counters are read together (one LDS round trip
      // instead of four), the decisions are then taken in order in registers, a later entry of the four
      // inheriting the state of an earlier one in the same row or column
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        unsigned int i[4], j[4], cc[4];
        mask_t rb[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const unsigned int idx = (pk[half * 2 + (k >> 1)] >> ((k & 1) * 16)) & (unsigned)(MM - 1);
          i[k] = idx / M;
          j[k] = idx % M;
          rb[k] = rowbits[i[k]][lane];
          cc[k] = colcnt[j[k]][lane];
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const unsigned int take = (mask_popc(rb[k]) < N && cc[k] < (unsigned)N) ? 1u : 0u;
          rb[k] |= (mask_t)take << j[k];
          cc[k] += take;
          placed += (int)take;
#pragma unroll
          for (int m = k + 1; m < 4; ++m) {
            rb[m] = i[m] == i[k] ? rb[k] : rb[m];
            cc[m] = j[m] == j[k] ? cc[k] : cc[m];
          }
        }
        // written back in order: for a row or column that occurs twice the later, more complete value stays
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          rowbits[i[k]][lane] = rb[k];
          colcnt[j[k]][lane] = (unsigned char)cc[k];
        }
      }
      }
#pragma unroll
      for (int d = 0; d < D; ++d) cur[d] = nxt[d];
    }
    for (int k = 0; k < M; ++k) rowmask[blk * M + k] = rowbits[k][lane];
    missing = need - placed;
  }
  if (batch.e[which].stats_out) {
    for (int s = 1; s < kWave; s <<= 1) missing += __shfl_xor(missing, s, kWave);
    if (lane == 0 && missing) atomicAdd(&hdr->stats[0], (unsigned long long)missing);
  }
}

// Ablation arm "Simple" (App. B.2.1): row-wise then column-wise N:M rounding of the plan.  In scan order
// (descending plan, ties by index) an entry survives the row stage while its row has passed fewer than N
// entries, and a survivor is kept while its column holds fewer than N: the first N of every row, then the
// first N survivors of every column.  One lane per block, same output as greedy_kernel.
template <int M>
__global__ __launch_bounds__(kWave) void simple_round_kernel(Batch batch) {
  using mask_t = block_mask_t<M>;
  constexpr int MM = M * M;
  __shared__ mask_t rowbits[M][kWave];
  __shared__ unsigned char passed[M][kWave], colcnt[M][kWave];
  const int which = find_problem(batch, blockIdx.x);
  const unsigned short* order = batch.e[which].order;
  const int64_t nblocks = batch.e[which].p.nblocks;
  const int N = batch.e[which].p.N;
  mask_t* rowmask = static_cast<mask_t*>(batch.e[which].rowmask);
  WsHeader* hdr = batch.e[which].hdr;
  const int lane = threadIdx.x;
  const int64_t blk = (int64_t)(blockIdx.x - batch.first[which]) * kWave + lane;
  for (int k = 0; k < M; ++k) {
    rowbits[k][lane] = 0;
    passed[k][lane] = 0;
    colcnt[k][lane] = 0;
  }
  int missing = 0;
  if (blk < nblocks) {
    const unsigned short* src = order + blk * MM;
    int placed = 0;
    for (int h = 0; h < MM; ++h) {
      const unsigned int idx = src[h] & (unsigned)(MM - 1);
      const unsigned int i = idx / M, j = idx % M;
      const unsigned int through = passed[i][lane];
      if (through < (unsigned)N) {
        passed[i][lane] = (unsigned char)(through + 1);
        const unsigned int cj = colcnt[j][lane];
        if (cj < (unsigned)N) {
          colcnt[j][lane] = (unsigned char)(cj + 1);
          rowbits[i][lane] |= (mask_t)1 << j;
          ++placed;
        }
      }
    }
    for (int k = 0; k < M; ++k) rowmask[blk * M + k] = rowbits[k][lane];
    missing = N * M - placed;
  }
  if (batch.e[which].stats_out) {
    for (int s = 1; s < kWave; s <<= 1) missing += __shfl_xor(missing, s, kWave);
    if (lane == 0 && missing) atomicAdd(&hdr->stats[0], (unsigned long long)missing);
  }
}

// LDS of the lane-parallel rounding steps for the G blocks a wave holds: the mask as row and column bit masks
// (rowm[r] bit c == colm[c] bit r == S[r][c]), column counters of the greedy selection, the importance block.
template <int M, int G>
struct RoundingLds {
  block_mask_t<M> rowm[G][M], colm[G][M];
  unsigned int colcnt[G][M];
  // (rows padded by one float: lane r reads row r, and with a row length of M every lane would hit the same bank)
  static constexpr int kImpLd = M + 1;
  float imp[G][M * kImpLd];
};

// The same selection with M lanes per block: the block's scan order is taken M entries at a time, one entry
// per lane, and all M are decided together.  An entry is rejected for certain when the entries before it in
// the chunk that are already accepted fill its row or its column, and accepted for certain when its row and
// its column have room even if every undecided entry before it were accepted; what is left undecided waits
// for the next round.  The earliest undecided entry of a block always resolves, so the rounds end, and by
// induction along the scan order every decision equals the sequential one.  Dependent chain: M chunks of a
// few rounds instead of M*M steps.
// A block owns LPB >= M consecutive lanes of the wave (LPB a power of two), of which the first M take part;
// fetch(pos) returns the flat index at scan position pos of this lane's block.  Leaves the mask in lds.rowm and
// returns the number of entries the lane's block holds.  To be called by whole single-wave workgroups.
template <int M, int LPB, class Fetch>
__device__ __forceinline__ int greedy_wide_scan(Fetch&& fetch, int N, int lane, RoundingLds<M, kWave / LPB>& lds) {
  using mask_t = block_mask_t<M>;
  constexpr int MM = M * M;
  constexpr int LOGM = M == 4 ? 2 : M == 8 ? 3 : M == 16 ? 4 : M == 32 ? 5 : 6;
  const int g = lane / LPB, ql = lane % LPB;
  const bool part = ql < M;
  if (part) {
    lds.rowm[g][ql] = 0;
    lds.colcnt[g][ql] = 0;
  }
  __syncthreads();
  const unsigned long long gmask = (M == 64 ? ~0ull : ((1ull << M) - 1)) << (g * LPB);
  const unsigned long long earlier = gmask & ((1ull << lane) - 1);  // lanes of this block before this one
  const int need = N * M;
  int placed = 0;
  unsigned int ahead = part ? fetch(ql) : 0u;
  for (int ch = 0; ch < M; ++ch) {
    const unsigned int idx = ahead & (unsigned)(MM - 1);
    if (ch + 1 < M && part) ahead = fetch((ch + 1) * M + ql);
    const unsigned int i = idx / M, j = idx % M;
    // lanes of this block whose entry lies in the same row / the same column
    unsigned long long same_row = gmask, same_col = gmask;
#pragma unroll
    for (int b = 0; b < LOGM; ++b) {
      const bool ib = (i >> b) & 1, jb = (j >> b) & 1;
      const unsigned long long rows_b = __ballot(ib), cols_b = __ballot(jb);
      same_row &= ib ? rows_b : ~rows_b;
      same_col &= jb ? cols_b : ~cols_b;
    }
    const unsigned long long before_row = same_row & earlier, before_col = same_col & earlier;
    const int room_row = N - mask_popc(lds.rowm[g][i]), room_col = N - (int)lds.colcnt[g][j];
    bool undecided = part && room_row > 0 && room_col > 0, take = false;
    unsigned long long taken = 0, open = __ballot(undecided);
    while (open) {
      if (undecided) {
        const int t_row = __popcll(taken & before_row), t_col = __popcll(taken & before_col);
        const int o_row = __popcll(open & before_row), o_col = __popcll(open & before_col);
        if (t_row >= room_row || t_col >= room_col) {
          undecided = false;
        } else if (t_row + o_row < room_row && t_col + o_col < room_col) {
          undecided = false;
          take = true;
        }
      }
      taken = __ballot(take);
      open = __ballot(undecided);
    }
    if (take) {
      atomicOr(&lds.rowm[g][i], (mask_t)1 << j);
      atomicAdd(&lds.colcnt[g][j], 1u);
    }
    placed += __popcll(taken & gmask);
    __syncthreads();
    if (!__any(placed < need)) break;  // every block of the wave is full
  }
  return placed;
}

template <int M>
__global__ __launch_bounds__(kWave) void greedy_wide_kernel(Batch batch) {
  using mask_t = block_mask_t<M>;
  constexpr int MM = M * M, G = kWave / M;
  __shared__ RoundingLds<M, G> lds;
  const int which = find_problem(batch, blockIdx.x);
  const unsigned short* order = batch.e[which].order;
  const int64_t nblocks = batch.e[which].p.nblocks;
  const int N = batch.e[which].p.N;
  mask_t* rowmask = static_cast<mask_t*>(batch.e[which].rowmask);
  WsHeader* hdr = batch.e[which].hdr;
  const int lane = threadIdx.x, g = lane / M, ql = lane % M;
  int64_t blk = (int64_t)(blockIdx.x - batch.first[which]) * G + g;
  const bool active = blk < nblocks;
  if (!active) blk = nblocks - 1;  // idle groups shadow the last block and write nothing
  const unsigned short* src = order + blk * MM;
  const int placed = greedy_wide_scan<M, M>([&](int pos) { return (unsigned int)src[pos]; }, N, lane, lds);
  if (active) rowmask[blk * M + ql] = lds.rowm[g][ql];
  if (batch.e[which].stats_out) {
    int missing = (active && ql == 0) ? N * M - placed : 0;
    for (int s = 1; s < kWave; s <<= 1) missing += __shfl_xor(missing, s, kWave);
    if (lane == 0 && missing) atomicAdd(&hdr->stats[0], (unsigned long long)missing);
  }
}

// Transpose of an M x M bit matrix held as one M-bit row per lane (M consecutive lanes): afterwards the
// lane that held row r holds column r.  log2(M) block-swap steps.
template <int M, int S = M / 2, class mask_t>
__device__ __forceinline__ mask_t bit_transpose(mask_t x, int ql) {
  if constexpr (S >= 1) {
    // bits whose index has bit S clear: S ones, S zeros, repeated
    mask_t lowpat = 0;
    for (int k = 0; k < M; ++k)
      if (!(k & S)) lowpat |= (mask_t)1 << k;
    mask_t other;
    if constexpr (sizeof(mask_t) == 8)
      other = (mask_t)__double_as_longlong(lane_xor<S>(__longlong_as_double((long long)x)));
    else
      other = (mask_t)lane_xor_i32<S>((int)x);
    x = (ql & S) ? (mask_t)((x & ~lowpat) | ((other & ~lowpat) >> S)) : (mask_t)((x & lowpat) | ((other & lowpat) << S));
    return bit_transpose<M, S / 2>(x, ql);
  } else {
    return x;
  }
}

// Best candidate of Eq. (5) held by a lane: score, flat index i'*M+j' (MM = none).  Higher score wins,
// equal scores go to the lower flat index.
struct SwapBest {
  double score;
  int arg;
};
template <int MM>
__device__ __forceinline__ SwapBest better_of(SwapBest a, SwapBest b) {
  const bool take_b = b.arg != MM && (a.arg == MM || b.score > a.score || (b.score == a.score && b.arg < a.arg));
  return take_b ? b : a;
}
template <int M, int STEP = 1>
__device__ __forceinline__ SwapBest group_best(SwapBest v) {
  if constexpr (STEP < M) {
    SwapBest o;
    o.score = lane_xor<STEP>(v.score);
    o.arg = lane_xor_i32<STEP>(v.arg);
    return group_best<M, STEP * 2>(better_of<M * M>(v, o));
  } else {
    return v;
  }
}

template <int M, int STEP = 1>
__device__ __forceinline__ double group_sum(double v) {
  if constexpr (STEP < M) {
    v += lane_xor<STEP>(v);
    return group_sum<M, STEP * 2>(v);
  } else {
    return v;
  }
}

// Algorithm 2 lines 7-13 and the mask write for the blocks of one wave.  A block owns LPB >= M consecutive lanes,
// of which the first M take part: lane r owns row r and column r of the block as bit masks.  On entry lds.rowm
// holds the mask greedy selection left.  blk: the lane's block (a valid one also for idle lanes, which write
// nothing: `active`).  To be called by whole single-wave workgroups.
template <int M, int LPB>
__device__ __forceinline__ void local_search_and_write(const DevProblem& p, const BatchEntry& e, int64_t blk, bool active,
                                                       int lane, RoundingLds<M, kWave / LPB>& lds) {
  using mask_t = block_mask_t<M>;
  constexpr int MM = M * M, LD = RoundingLds<M, kWave / LPB>::kImpLd;
  uint8_t* mask = e.mask;
  WsHeader* hdr = e.hdr;
  const int wide_store = e.wide_store;
  double* block_objective = e.block_objective;
  const uint8_t* prev_mask = e.prev_mask;
  const bool want_stats = e.stats_out != nullptr;
  const int g = lane / LPB, ql = lane % LPB;
  const bool part = ql < M;
  const int qm = ql % M;  // (an index that stays inside the block's LDS rows also for the lanes that only tag along)
  const int64_t r0 = (blk / p.bc) * M, c0 = (blk % p.bc) * M;
  const mask_t one = 1;

  // the transpose of the mask greedy selection left
  {
    const mask_t r = part ? lds.rowm[g][qm] : (mask_t)0;
    const mask_t c = bit_transpose<M>(r, qm);
    if (part) lds.colm[g][qm] = c;
  }
  __syncthreads();
  const auto popc = [](mask_t v) { return mask_popc(v); };
  const unsigned long long gmask = (M == 64 ? ~0ull : ((1ull << M) - 1)) << (g * LPB);
  const bool any_short = __any(part && popc(lds.rowm[g][qm]) < p.N);
  if ((any_short || block_objective) && part) {
    // local search scores on the importance (Eq. 5), staged in LDS: this lane fetches column ql of its
    // block, all M loads in flight at once
    float col[M];
    block_column_importance<M>(p, r0, c0 + qm, col);
#pragma unroll
    for (int k = 0; k < M; ++k) lds.imp[g][k * LD + qm] = col[k];
  }
  __syncthreads();

  int rounds = 0, nonpos = 0;
  bool open = any_short;  // this block may still take swaps
  while (any_short) {
    const mask_t Srow = part ? lds.rowm[g][qm] : (mask_t)0;
    const mask_t Scol = part ? lds.colm[g][qm] : (mask_t)0;
    const unsigned long long rb = __ballot(part && popc(Srow) < p.N) & gmask;
    const unsigned long long cb = __ballot(part && popc(Scol) < p.N) & gmask;
    if (rb == 0 || cb == 0 || (p.strict && rounds >= p.L)) open = false;
    if (!__any(open)) break;
    // line 10: the lowest-index row i and column j that are short
    const int i = open ? (__ffsll((long long)rb) - 1 - g * LPB) : 0;
    const int j = open ? (__ffsll((long long)cb) - 1 - g * LPB) : 0;
    // line 11 for i' = this lane: columns j' with S[i'][j'] = 1 and S[i][j'] = 0, provided S[i'][j] = 0
    mask_t cand = Srow & ~lds.rowm[g][i];
    if (!open || !part || ((lds.colm[g][j] >> qm) & 1)) cand = 0;
    const double base = (double)lds.imp[g][qm * LD + j];
    SwapBest best = {-std::numeric_limits<double>::infinity(), MM};
    while (__any(cand != 0)) {
      if (cand != 0) {
        const int jp = sizeof(mask_t) == 8 ? __ffsll((long long)cand) - 1 : __ffs((int)cand) - 1;
        cand &= cand - 1;
        const double sc = ((double)lds.imp[g][i * LD + jp] + base) - (double)lds.imp[g][qm * LD + jp];
        if (best.arg == MM || sc > best.score) {
          best.score = sc;
          best.arg = qm * M + jp;
        }
      }
    }
    best = group_best<M>(best);
    if (open) ++rounds;
    bool apply = open && best.arg != MM;
    if (p.strict && !(best.score > 0.0)) apply = false;
    if (open && !apply) open = false;  // nothing changes any more for this block
    __syncthreads();
    if (apply && ql == 0) {
      // line 13: remove (i', j'), insert (i', j) and (i, j')
      const int ip = best.arg / M, jp = best.arg % M;
      lds.rowm[g][ip] = (lds.rowm[g][ip] & ~(one << jp)) | (one << j);
      lds.rowm[g][i] |= one << jp;
      lds.colm[g][jp] = (lds.colm[g][jp] & ~(one << ip)) | (one << i);
      lds.colm[g][j] |= one << ip;
      if (!(best.score > 0.0)) ++nonpos;
    }
    __syncthreads();
  }

  if (active && part) {
    const mask_t bits = lds.rowm[g][qm];
    uint8_t* dst = mask + (r0 + qm) * p.cols + c0;
    if (wide_store) {
      // 4 mask bytes per 32-bit word: bit k of a nibble goes to byte k
      unsigned int w[M / 4];
#pragma unroll
      for (int k = 0; k < M / 4; ++k) w[k] = (((unsigned int)(bits >> (4 * k)) & 0xFu) * 0x00204081u) & 0x01010101u;
      if constexpr (M == 4) {
        *reinterpret_cast<unsigned int*>(dst) = w[0];
      } else if constexpr (M == 8) {
        *reinterpret_cast<uint2*>(dst) = make_uint2(w[0], w[1]);
      } else {
#pragma unroll
        for (int k = 0; k < M / 16; ++k)
          reinterpret_cast<uint4*>(dst)[k] = make_uint4(w[4 * k], w[4 * k + 1], w[4 * k + 2], w[4 * k + 3]);
      }
    } else {
      for (int k = 0; k < M; ++k) dst[k] = (uint8_t)((bits >> k) & 1);
    }
  }
  if (block_objective) {
    // sum S * importance of this block for the mask found and for the caller's previous mask: every lane
    // sums its row left to right, the rows are then added in a fixed butterfly order
    double mine = 0.0, theirs = 0.0;
    if (part) {
      const mask_t bits = lds.rowm[g][qm];
      mask_t prev_bits = 0;
      if (prev_mask) {
        // the previous mask's row as bits: the byte loads are independent of each other
        const uint8_t* prev = prev_mask + (r0 + qm) * p.cols + c0;
        uint8_t pm[M];
#pragma unroll
        for (int k = 0; k < M; ++k) pm[k] = prev[k];
#pragma unroll
        for (int k = 0; k < M; ++k) prev_bits |= (mask_t)(pm[k] != 0) << k;
      }
#pragma unroll
      for (int k = 0; k < M; ++k) {
        const double v = (double)lds.imp[g][qm * LD + k];
        mine += ((bits >> k) & 1) ? v : 0.0;
        theirs += ((prev_bits >> k) & 1) ? v : 0.0;
      }
    }
    mine = group_sum<M>(mine);
    theirs = group_sum<M>(theirs);
    if (active && ql == 0) {
      block_objective[2 * blk] = mine;
      block_objective[2 * blk + 1] = theirs;
    }
  }
  if (want_stats && active && part) {
    const int left = p.N - popc(lds.rowm[g][qm]);
    if (left) atomicAdd(&hdr->stats[3], (unsigned long long)left);
    if (ql == 0) {
      if (nonpos) atomicAdd(&hdr->stats[1], (unsigned long long)nonpos);
      if (!p.strict && rounds > p.L) atomicAdd(&hdr->stats[2], 1ull);
    }
  }
}

// The stand-alone kernel: M lanes per block, 64/M blocks per wave, one wave per workgroup; the mask greedy
// selection left comes from the workspace.
template <int M>
__global__ __launch_bounds__(kWave) void finalize_kernel(Batch batch) {
  using mask_t = block_mask_t<M>;
  constexpr int G = kWave / M;
  __shared__ RoundingLds<M, G> lds;
  const int which = find_problem(batch, blockIdx.x);
  const DevProblem p = batch.e[which].p;
  const mask_t* rowmask = static_cast<const mask_t*>(batch.e[which].rowmask);
  const int lane = threadIdx.x, g = lane / M, ql = lane % M;
  int64_t blk = (int64_t)(blockIdx.x - batch.first[which]) * G + g;
  const bool active = blk < p.nblocks;
  if (!active) blk = p.nblocks - 1;  // idle groups shadow the last block and write nothing
  lds.rowm[g][ql] = rowmask[blk * M + ql];
  local_search_and_write<M, M>(p, batch.e[which], blk, active, lane, lds);
}

}  // namespace tsenor_dev
