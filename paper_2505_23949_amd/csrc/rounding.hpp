// Algorithm 2: greedy selection (one lane per block) and local search plus the mask write.
#pragma once
#include <limits>

#include "lanes.hpp"
#include "problem.hpp"

namespace tsenor_dev {

// Algorithm 2 lines 1-6: scan the entries of a block in sorted order and keep an entry while its row
// and its column hold fewer than N.  One lane per block; bit t of the output says whether the t-th
// entry of the order was kept.
template <int M>
__global__ __launch_bounds__(kWave) void greedy_kernel(const unsigned short* order, int64_t nblocks, int N,
                                                       unsigned int* accept, WsHeader* hdr) {
  constexpr int MM = M * M, WORDS = MM >= 32 ? MM / 32 : 1, PER_WORD = MM >= 32 ? 32 : MM;
  __shared__ unsigned char cnt[2 * M][kWave];
  const int lane = threadIdx.x;
  const int64_t blk = (int64_t)blockIdx.x * kWave + lane;
  for (int k = 0; k < 2 * M; ++k) cnt[k][lane] = 0;
  int missing = 0;
  if (blk < nblocks) {
    const unsigned short* src = order + blk * MM;
    int placed = 0;
    for (int w = 0; w < WORDS; ++w) {
      unsigned int acc = 0;
      for (int h = 0; h < PER_WORD; h += 8) {
        const uint4 v = *reinterpret_cast<const uint4*>(src + w * PER_WORD + h);
        const unsigned int pk[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const unsigned int idx = (pk[u >> 1] >> ((u & 1) * 16)) & (unsigned)(MM - 1);
          const unsigned int i = idx / M, j = idx % M;
          const unsigned int ri = cnt[i][lane], cj = cnt[M + j][lane];
          if (ri < (unsigned)N && cj < (unsigned)N) {
            cnt[i][lane] = (unsigned char)(ri + 1);
            cnt[M + j][lane] = (unsigned char)(cj + 1);
            acc |= 1u << (h + u);
            ++placed;
          }
        }
      }
      accept[blk * WORDS + w] = acc;
    }
    missing = N * M - placed;
  }
  for (int s = 1; s < kWave; s <<= 1) missing += __shfl_xor(missing, s, kWave);
  if (lane == 0 && missing) atomicAdd(&hdr->stats[0], (unsigned long long)missing);
}

// Algorithm 2 lines 7-13 and the mask write.  L3 lanes per block (M <= L3 <= 64), 64/L3 blocks per wave.
template <int M, int L3>
__global__ __launch_bounds__(kWave) void finalize_kernel(DevProblem p, const unsigned short* order,
                                                         const unsigned int* accept, uint8_t* mask, WsHeader* hdr,
                                                         int64_t* stats_out) {
  constexpr int MM = M * M, G = kWave / L3, WORDS = MM >= 32 ? MM / 32 : 1, PER_WORD = MM >= 32 ? 32 : MM;
  static_assert(L3 >= M && kWave % L3 == 0 && MM % L3 == 0, "lanes per block");
  __shared__ float imp[G][MM];
  __shared__ unsigned char S[G][MM];
  __shared__ int Rc[G][M], Cc[G][M];
  const int lane = threadIdx.x, g = lane / L3, ql = lane % L3;
  int64_t blk = (int64_t)blockIdx.x * G + g;
  const bool active = blk < p.nblocks;
  if (!active) blk = p.nblocks - 1;
  const int64_t r0 = (blk / p.bc) * M, c0 = (blk % p.bc) * M;

  for (int e = ql; e < MM; e += L3) {
    imp[g][e] = load_importance(p, r0 + e / M, c0 + e % M);
    S[g][e] = 0;
  }
  __syncthreads();
  for (int pos = ql; pos < MM; pos += L3) {
    const unsigned int bit = (accept[blk * WORDS + pos / PER_WORD] >> (pos % PER_WORD)) & 1u;
    if (bit) S[g][order[blk * MM + pos] & (MM - 1)] = 1;
  }
  __syncthreads();
  if (ql < M) {
    int r = 0, c = 0;
    for (int k = 0; k < M; ++k) {
      r += S[g][ql * M + k];
      c += S[g][k * M + ql];
    }
    Rc[g][ql] = r;
    Cc[g][ql] = c;
  }
  __syncthreads();

  const unsigned long long gmask = (L3 == 64 ? ~0ull : ((1ull << L3) - 1)) << (g * L3);
  int rounds = 0, nonpos = 0;
  bool open = true;  // this block may still take swaps
  for (;;) {
    const bool rdef = ql < M && Rc[g][ql < M ? ql : 0] < p.N;
    const bool cdef = ql < M && Cc[g][ql < M ? ql : 0] < p.N;
    const unsigned long long rb = __ballot(rdef) & gmask, cb = __ballot(cdef) & gmask;
    if (rb == 0 || cb == 0 || (p.strict && rounds >= p.L)) open = false;
    if (!__any(open)) break;
    // Pick i, j: the lowest-index row and column that are short (line 10)
    const int i = open ? (__ffsll((long long)rb) - 1 - g * L3) : 0;
    const int j = open ? (__ffsll((long long)cb) - 1 - g * L3) : 0;
    // line 11: arg max of Eq. (5) over valid (i', j'); ties to the lowest flat index
    double best = -std::numeric_limits<double>::infinity();
    int arg = MM;
    if (open) {
      for (int e = ql; e < MM; e += L3) {
        const int ip = e / M, jp = e % M;
        if (S[g][e] && !S[g][i * M + jp] && !S[g][ip * M + j]) {
          const double sc = (double)imp[g][i * M + jp] + (double)imp[g][ip * M + j] - (double)imp[g][e];
          if (arg == MM || sc > best) {
            best = sc;
            arg = e;
          }
        }
      }
    }
#pragma unroll
    for (int m = 1; m < L3; m <<= 1) {
      const double ob = __shfl_xor(best, m, kWave);
      const int oa = __shfl_xor(arg, m, kWave);
      if (oa != MM && (arg == MM || ob > best || (ob == best && oa < arg))) {
        best = ob;
        arg = oa;
      }
    }
    if (open) ++rounds;
    bool apply = open && arg != MM;
    if (p.strict && !(best > 0.0)) apply = false;
    if (open && !apply) open = false;  // nothing changes any more for this block
    __syncthreads();
    if (apply && ql == 0) {
      // line 13: remove (i', j'), insert (i', j) and (i, j')
      const int ip = arg / M, jp = arg % M;
      S[g][arg] = 0;
      S[g][ip * M + j] = 1;
      S[g][i * M + jp] = 1;
      Rc[g][i] += 1;
      Cc[g][j] += 1;
      if (!(best > 0.0)) ++nonpos;
    }
    __syncthreads();
  }

  if (active) {
    for (int e = ql; e < MM; e += L3) mask[(r0 + e / M) * p.cols + c0 + e % M] = S[g][e];
    if (ql == 0) {
      int left = 0;
      for (int k = 0; k < M; ++k) left += p.N - Rc[g][k];
      if (nonpos) atomicAdd(&hdr->stats[1], (unsigned long long)nonpos);
      if (!p.strict && rounds > p.L) atomicAdd(&hdr->stats[2], 1ull);
      if (left) atomicAdd(&hdr->stats[3], (unsigned long long)left);
    }
  }
  (void)stats_out;
}

}  // namespace tsenor_dev
