// Transposable N:M mask finder for MI355X (gfx950): kernels and C ABI.
//
// One call enqueues, on the caller's stream:
//   1. init_kernel / absmax_kernel      importance maximum of the matrix (REL_MATRIX_MAX tau only)
//   2. dykstra_sort_kernel              tile load, all T Dykstra iterations of Algorithm 1 on chip,
//                                       sort of the M*M plan entries of every block; writes the greedy
//                                       scan order (and the plan if asked for)
//   3. greedy_kernel                    Algorithm 2 lines 1-6, one lane per block
//   4. finalize_kernel                  Algorithm 2 lines 7-13 (local search) and the mask write
//
// How Algorithm 1 is evaluated.  With A = log S + log Q, the cap step gives log S = min(A, 0) and
// log Q = max(A, 0) after every iteration, and one iteration adds a row term and a column term to A.
// So A = K + f_i + g_j with K = tau_eff * importance, and the whole Dykstra state of a block is K
// plus 2M potentials.  The kernel keeps kappa = exp(K - max K) and the scalings U_i = exp(f_i),
// V_j = exp(g_j) in double precision and iterates
//     e_ij = min(kappa_ij V_j U_i, 1);  R_i = N / sum_j e_ij;  C_j = N / sum_i e_ij R_i;
//     U_i *= R_i;  V_j *= C_j
// which is Algorithm 1 lines 3-6 in exact arithmetic (the row scaling is applied after the cap of
// the previous iteration, exactly as in the listing of App. A.2).  Four multiply/add per entry and
// iteration, no transcendental in the loop; MI355X issues double-precision vector operations at the
// same rate as single-precision ones, and doubles make the result agree with a double-precision
// reference to ~1e-13, so the sort order below is decided on the same numbers.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cmath>
#include <limits>

#include "tsenor.h"

namespace {

constexpr int kWave = 64;
constexpr double kMinLogKernel = -700.0;  // exp(-700) is still a normal double
constexpr int kIdxBits = 12;              // flat index within a block: up to 64*64 entries

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

__device__ __forceinline__ double tau_eff_of(const DevProblem& p, const WsHeader* hdr) {
  if (p.tau_mode == TSENOR_TAU_ABSOLUTE) return p.tau;
  float mx = __uint_as_float(hdr->max_bits);
  return mx > 0.0f ? 1.0 / (p.tau * (double)mx) : 0.0;
}

__global__ void init_kernel(WsHeader* hdr) {
  hdr->max_bits = 0u;
  hdr->pad = 0u;
  hdr->tau_eff = 0.0;
  for (int k = 0; k < 4; ++k) hdr->stats[k] = 0ull;
}

// Largest importance of the matrix (App. B.1 parameter choice, relative tau).
__global__ __launch_bounds__(256) void absmax_kernel(DevProblem p, int64_t rows, WsHeader* hdr) {
  const int64_t total = rows * p.cols;
  float m = 0.0f;
  for (int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; k < total; k += (int64_t)gridDim.x * blockDim.x) {
    float v = load_importance(p, k / p.cols, k % p.cols);
    m = fmaxf(m, v);
  }
  for (int s = 1; s < kWave; s <<= 1) m = fmaxf(m, __shfl_xor(m, s, kWave));
  if ((threadIdx.x & (kWave - 1)) == 0) atomicMax(&hdr->max_bits, __float_as_uint(m));
}

__global__ void fill_kernel(uint8_t* mask, int64_t total, uint8_t value) {
  for (int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; k < total; k += (int64_t)gridDim.x * blockDim.x)
    mask[k] = value;
}

// 1/d to double precision: hardware estimate plus two Newton steps.
__device__ __forceinline__ double fast_rcp(double d) {
  double x = __builtin_amdgcn_rcp(d);
  x = fma(fma(-d, x, 1.0), x, x);
  x = fma(fma(-d, x, 1.0), x, x);
  return x;
}

template <int FIRST, int LAST>  // sum over the lanes that differ in the bits FIRST..LAST (masks, powers of two)
__device__ __forceinline__ double allreduce_sum(double v) {
#pragma unroll
  for (int m = FIRST; m <= LAST; m <<= 1) v += __shfl_xor(v, m, kWave);
  return v;
}

template <int FIRST, int LAST>
__device__ __forceinline__ double allreduce_max(double v) {
#pragma unroll
  for (int m = FIRST; m <= LAST; m <<= 1) v = fmax(v, __shfl_xor(v, m, kWave));
  return v;
}

__device__ __forceinline__ void compare_exchange(double& lo, double& hi) {
  double a = fmin(lo, hi), b = fmax(lo, hi);
  lo = a;
  hi = b;
}

// Ascending bitonic sort of E*LPB distinct positive doubles spread over LPB lanes (position q*E + r).
// Every merge starts with the mirrored compare (p against p ^ (k-1)) so that the smaller key always
// goes to the lower position and no direction flags are needed.
template <int E, int LPB>
__device__ __forceinline__ void sort_ascending(double (&c)[E], int q) {
  constexpr int NTOT = E * LPB;
#pragma unroll
  for (int k = 2; k <= NTOT; k <<= 1) {
    if (k <= E) {
#pragma unroll
      for (int r = 0; r < E; ++r) {
        const int pr = r ^ (k - 1);
        if (pr > r) compare_exchange(c[r], c[pr]);
      }
    } else {
      const int lm = k / E - 1;
      const bool keep_min = (q & (k / E / 2)) == 0;
      double o[E];
#pragma unroll
      for (int r = 0; r < E; ++r) o[r] = __shfl_xor(c[E - 1 - r], lm, kWave);
#pragma unroll
      for (int r = 0; r < E; ++r) c[r] = ((c[r] < o[r]) == keep_min) ? c[r] : o[r];
    }
#pragma unroll
    for (int j = k >> 2; j > 0; j >>= 1) {
      if (j < E) {
#pragma unroll
        for (int r = 0; r < E; ++r) {
          const int pr = r ^ j;
          if (pr > r) compare_exchange(c[r], c[pr]);
        }
      } else {
        const int lm = j / E;
        const bool keep_min = (q & lm) == 0;
#pragma unroll
        for (int r = 0; r < E; ++r) {
          double o = __shfl_xor(c[r], lm, kWave);
          c[r] = ((c[r] < o) == keep_min) ? c[r] : o;
        }
      }
    }
  }
}

// Tile load, Algorithm 1, sort.  A block is spread over LPB = GY*GX lanes as a GY x GX grid of
// TH x TW tiles; a wave holds 64/LPB blocks.  STORE_E keeps the capped entries of the row pass in
// registers for the column pass; without it they are recomputed (for tiles too large to hold twice).
template <int M, int GY, int GX, bool STORE_E>
__global__ __launch_bounds__(256) void dykstra_sort_kernel(DevProblem p, WsHeader* hdr, unsigned short* order,
                                                            double* plan_out, double* tau_eff_out) {
  constexpr int TH = M / GY, TW = M / GX, LPB = GY * GX, BPW = kWave / LPB, E = TH * TW;
  static_assert(M % GY == 0 && M % GX == 0 && kWave % LPB == 0, "tiling must divide");
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t wave = (int64_t)blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave);
  const int q = lane % LPB, gx = q % GX, gy = q / GX;
  int64_t blk = wave * BPW + lane / LPB;
  const bool active = blk < p.nblocks;
  if (!active) blk = p.nblocks - 1;  // idle lanes shadow the last block and write nothing
  const int64_t r0 = (blk / p.bc) * M, c0 = (blk % p.bc) * M;
  const double tau_eff = tau_eff_of(p, hdr);
  if (tau_eff_out && blockIdx.x == 0 && threadIdx.x == 0) *tau_eff_out = tau_eff;

  // in-kernel coordinates (ri, cj); with `transpose` they are (column, row) of the matrix block, which
  // turns "rows first" into "columns first" (TSENOR_FLAG_COLS_FIRST)
  auto mat_row = [&](int ri, int cj) { return p.transpose ? cj : ri; };
  auto mat_col = [&](int ri, int cj) { return p.transpose ? ri : cj; };

  double kap[TH][TW];
  double mx = 0.0;
#pragma unroll
  for (int a = 0; a < TH; ++a)
#pragma unroll
    for (int b = 0; b < TW; ++b) {
      const int ri = gy * TH + a, cj = gx * TW + b;
      const float imp = load_importance(p, r0 + mat_row(ri, cj), c0 + mat_col(ri, cj));
      kap[a][b] = tau_eff * (double)imp;  // K of Algorithm 1 line 1
      mx = fmax(mx, kap[a][b]);
    }
  mx = allreduce_max<1, LPB / 2>(mx);

  double c[E];  // sort keys
  if (p.T == 0) {
    // no iterations: the greedy order is descending K itself
#pragma unroll
    for (int a = 0; a < TH; ++a)
#pragma unroll
      for (int b = 0; b < TW; ++b) {
        const int ri = gy * TH + a, cj = gx * TW + b;
        const unsigned long long idx = (unsigned long long)(mat_row(ri, cj) * M + mat_col(ri, cj));
        const unsigned long long bits = (unsigned long long)__double_as_longlong(kap[a][b]);
        const unsigned long long key = (0x40A0000000000000ull - bits) & ~((1ull << kIdxBits) - 1);
        c[a * TW + b] = __longlong_as_double((long long)(key | idx));
        if (plan_out && active)
          plan_out[(r0 + mat_row(ri, cj)) * p.cols + c0 + mat_col(ri, cj)] = exp(kap[a][b]);
      }
  } else {
#pragma unroll
    for (int a = 0; a < TH; ++a)
#pragma unroll
      for (int b = 0; b < TW; ++b) kap[a][b] = exp(fmax(kap[a][b] - mx, kMinLogKernel));

    const double Nd = (double)p.N;
    double U[TH], V[TW];
#pragma unroll
    for (int a = 0; a < TH; ++a) U[a] = 1.0;
#pragma unroll
    for (int b = 0; b < TW; ++b) V[b] = 1.0;

    for (int t = 0; t < p.T; ++t) {
      double e[STORE_E ? TH : 1][STORE_E ? TW : 1];
      double R[TH];
      // projection onto C1 (Algorithm 1 line 3) applied to the capped plan of the previous iteration
#pragma unroll
      for (int a = 0; a < TH; ++a) {
        double s = 0.0;
#pragma unroll
        for (int b = 0; b < TW; ++b) {
          const double ev = fmin(fmax((kap[a][b] * V[b]) * U[a], 0.0), 1.0);
          if constexpr (STORE_E) e[a][b] = ev;
          s += ev;
        }
        R[a] = s;
      }
#pragma unroll
      for (int a = 0; a < TH; ++a) {
        const double s = fmax(allreduce_sum<1, GX / 2>(R[a]), 1e-300);
        R[a] = Nd * fast_rcp(s);
      }
      // projection onto C2 (line 4)
      double C[TW];
#pragma unroll
      for (int b = 0; b < TW; ++b) {
        double s = 0.0;
#pragma unroll
        for (int a = 0; a < TH; ++a) {
          double ev;
          if constexpr (STORE_E)
            ev = e[a][b];
          else
            ev = fmin(fmax((kap[a][b] * V[b]) * U[a], 0.0), 1.0);
          s = fma(ev, R[a], s);
        }
        C[b] = s;
      }
#pragma unroll
      for (int b = 0; b < TW; ++b) {
        const double s = fmax(allreduce_sum<GX, LPB / 2>(C[b]), 1e-300);
        V[b] *= Nd * fast_rcp(s);
      }
#pragma unroll
      for (int a = 0; a < TH; ++a) U[a] *= R[a];
      // lines 5-6 (cap and dual) are the min(., 1) at the top of the next pass
    }

    double lu[TH], lv[TW];
#pragma unroll
    for (int a = 0; a < TH; ++a) lu[a] = log(U[a]);
#pragma unroll
    for (int b = 0; b < TW; ++b) lv[b] = log(V[b]);
#pragma unroll
    for (int a = 0; a < TH; ++a)
#pragma unroll
      for (int b = 0; b < TW; ++b) {
        const int ri = gy * TH + a, cj = gx * TW + b;
        const int64_t mr = r0 + mat_row(ri, cj), mc = c0 + mat_col(ri, cj);
        const double K = tau_eff * (double)load_importance(p, mr, mc);
        // log S^(T) = min(K + f_i + g_j, 0)
        const double key = fmin(fmax(K - mx, kMinLogKernel) + (lu[a] + lv[b]), 0.0);
        if (plan_out && active) plan_out[mr * p.cols + mc] = exp(key);
        const unsigned long long idx = (unsigned long long)(mat_row(ri, cj) * M + mat_col(ri, cj));
        const unsigned long long bits = (unsigned long long)__double_as_longlong(fabs(key));
        // descending key, ties by ascending flat index; + 2^52 keeps the pattern a normal double
        c[a * TW + b] =
            __longlong_as_double((long long)(((bits & ~((1ull << kIdxBits) - 1)) | idx) + (1ull << 52)));
      }
  }

  sort_ascending<E, LPB>(c, q);

  if (active) {
    unsigned short* dst = order + blk * (int64_t)(M * M) + q * E;
#pragma unroll
    for (int r = 0; r < E; ++r)
      dst[r] = (unsigned short)((unsigned long long)__double_as_longlong(c[r]) & ((1ull << kIdxBits) - 1));
  }
}

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

__global__ void stats_kernel(const WsHeader* hdr, int64_t* stats_out) {
  for (int k = 0; k < 4; ++k) stats_out[k] = (int64_t)hdr->stats[k];
}

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct WsLayout {
  size_t header, order, accept, total;
};

inline int words_per_block(int M) { return M * M >= 32 ? M * M / 32 : 1; }

WsLayout layout_of(const tsenor_problem& p) {
  WsLayout l;
  const size_t elems = (size_t)p.rows * (size_t)p.cols;
  const size_t nblocks = elems / ((size_t)p.M * p.M);
  l.header = 0;
  l.order = kAlign;
  l.accept = l.order + align_up(elems * sizeof(unsigned short));
  l.total = l.accept + align_up(nblocks * words_per_block(p.M) * sizeof(unsigned int));
  return l;
}

int validate(const tsenor_problem* p) {
  if (!p || !p->W || !p->mask) return TSENOR_ERR_NULL;
  if (p->M != 4 && p->M != 8 && p->M != 16 && p->M != 32 && p->M != 64) return TSENOR_ERR_UNSUPPORTED;
  if (p->dtype != TSENOR_F32 && p->dtype != TSENOR_BF16) return TSENOR_ERR_UNSUPPORTED;
  if (p->tau_mode != TSENOR_TAU_ABSOLUTE && p->tau_mode != TSENOR_TAU_REL_MATRIX_MAX) return TSENOR_ERR_UNSUPPORTED;
  if (p->flags & ~(uint32_t)(TSENOR_FLAG_STRICT_PAPER | TSENOR_FLAG_COLS_FIRST)) return TSENOR_ERR_UNSUPPORTED;
  if (p->rows <= 0 || p->cols <= 0 || p->rows % p->M || p->cols % p->M || p->ld < p->cols) return TSENOR_ERR_SHAPE;
  if (p->rows > (int64_t)1 << 31 || p->cols > (int64_t)1 << 31 || p->rows * p->cols > (int64_t)1 << 40)
    return TSENOR_ERR_SHAPE;
  if (p->N < 0 || p->N > p->M) return TSENOR_ERR_NM;
  if (!(p->tau > 0.0) || !std::isfinite(p->tau) || p->iters < 0 || p->local_search_steps < 0) return TSENOR_ERR_PARAM;
  if (p->tau_mode == TSENOR_TAU_REL_MATRIX_MAX && p->tau < 1.0 / 690.0) return TSENOR_ERR_PARAM;
  return TSENOR_OK;
}

template <int M, int GY, int GX, bool STORE_E, int L3>
int launch_all(const DevProblem& dp, int64_t rows, const tsenor_problem& p, char* ws, const WsLayout& l,
               hipStream_t stream) {
  WsHeader* hdr = reinterpret_cast<WsHeader*>(ws + l.header);
  unsigned short* order = reinterpret_cast<unsigned short*>(ws + l.order);
  unsigned int* accept = reinterpret_cast<unsigned int*>(ws + l.accept);
  init_kernel<<<1, 1, 0, stream>>>(hdr);
  if (dp.tau_mode == TSENOR_TAU_REL_MATRIX_MAX) {
    const int64_t total = rows * dp.cols;
    const int grid = (int)std::min<int64_t>((total + 256 * 8 - 1) / (256 * 8), 256 * 16);
    absmax_kernel<<<grid, 256, 0, stream>>>(dp, rows, hdr);
  }
  constexpr int BPW = kWave / (GY * GX);
  const int64_t waves = (dp.nblocks + BPW - 1) / BPW;
  dykstra_sort_kernel<M, GY, GX, STORE_E>
      <<<(unsigned)((waves + 3) / 4), 256, 0, stream>>>(dp, hdr, order, p.plan_out, p.tau_eff_out);
  greedy_kernel<M><<<(unsigned)((dp.nblocks + kWave - 1) / kWave), kWave, 0, stream>>>(order, dp.nblocks, dp.N,
                                                                                      accept, hdr);
  constexpr int G = kWave / L3;
  finalize_kernel<M, L3>
      <<<(unsigned)((dp.nblocks + G - 1) / G), kWave, 0, stream>>>(dp, order, accept, p.mask, hdr, p.stats_out);
  if (p.stats_out) stats_kernel<<<1, 1, 0, stream>>>(hdr, p.stats_out);
  return hipGetLastError() == hipSuccess ? TSENOR_OK : TSENOR_ERR_HIP;
}

int run_one(const tsenor_problem& p, char* ws, hipStream_t stream) {
  const int64_t total = p.rows * p.cols;
  if (p.N == 0 || p.N == p.M) {
    const int grid = (int)std::min<int64_t>((total + 255) / 256, 65535);
    fill_kernel<<<grid, 256, 0, stream>>>(p.mask, total, p.N == 0 ? 0 : 1);
    // the plan of a degenerate problem is the mask itself; stats are zero
    if (p.stats_out || p.tau_eff_out || p.plan_out) {
      WsHeader* hdr = reinterpret_cast<WsHeader*>(ws);
      init_kernel<<<1, 1, 0, stream>>>(hdr);
      if (p.stats_out) stats_kernel<<<1, 1, 0, stream>>>(hdr, p.stats_out);
    }
    return hipGetLastError() == hipSuccess ? TSENOR_OK : TSENOR_ERR_HIP;
  }
  DevProblem dp;
  dp.W = p.W;
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
  dp.tau = p.tau;
  dp.tau_mode = p.tau_mode;
  const WsLayout l = layout_of(p);
  switch (p.M) {
    case 4: return launch_all<4, 1, 1, true, 16>(dp, p.rows, p, ws, l, stream);
    case 8: return launch_all<8, 2, 2, true, 64>(dp, p.rows, p, ws, l, stream);
    case 16: return launch_all<16, 4, 4, true, 64>(dp, p.rows, p, ws, l, stream);
    case 32: return launch_all<32, 4, 8, true, 64>(dp, p.rows, p, ws, l, stream);
    case 64: return launch_all<64, 8, 8, false, 64>(dp, p.rows, p, ws, l, stream);
  }
  return TSENOR_ERR_UNSUPPORTED;
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
  if (!problems || count <= 0) return TSENOR_ERR_NULL;
  size_t need = 0;
  for (int k = 0; k < count; ++k) {
    const int rc = validate(&problems[k]);
    if (rc != TSENOR_OK) return rc;
    need += layout_of(problems[k]).total;
  }
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % kAlign) || workspace_bytes < need)
    return TSENOR_ERR_WORKSPACE;
  char* ws = static_cast<char*>(workspace);
  for (int k = 0; k < count; ++k) {
    const int rc = run_one(problems[k], ws, static_cast<hipStream_t>(stream));
    if (rc != TSENOR_OK) return rc;
    ws += layout_of(problems[k]).total;
  }
  return TSENOR_OK;
}

int tsenor_mask_ex(const tsenor_problem* p, void* workspace, size_t workspace_bytes, tsenor_stream_t stream) {
  return tsenor_mask_batched(p, 1, workspace, workspace_bytes, stream);
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
  const int rc2 = run_one(p, static_cast<char*>(ws), s);
  if (hipFreeAsync(ws, s) != hipSuccess) return TSENOR_ERR_HIP;
  return rc2;
}

const char* tsenor_status_string(int status) {
  switch (status) {
    case TSENOR_OK: return "ok";
    case TSENOR_ERR_NULL: return "a required pointer is NULL";
    case TSENOR_ERR_SHAPE: return "rows/cols must be positive multiples of M, ld >= cols, at most 2^40 weights";
    case TSENOR_ERR_NM: return "N must satisfy 0 <= N <= M";
    case TSENOR_ERR_UNSUPPORTED: return "unsupported M (4, 8, 16, 32, 64), dtype, tau_mode or flag";
    case TSENOR_ERR_PARAM: return "tau must be finite and > 0 (>= 1/690 in REL_MATRIX_MAX mode), iters and local_search_steps >= 0";
    case TSENOR_ERR_WORKSPACE: return "workspace is NULL, not 256-byte aligned or smaller than tsenor_workspace_bytes";
    case TSENOR_ERR_HIP: return "a HIP call failed";
  }
  return "unknown status";
}

int tsenor_version(void) { return 100; }

}  // extern "C"
