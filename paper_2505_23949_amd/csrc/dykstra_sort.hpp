// Tile load, Algorithm 1 (Dykstra iterations) and the sort that feeds Algorithm 2, one kernel.
//
// How Algorithm 1 is evaluated.  With A = log S + log Q, the cap step (lines 5-6) gives
// log S = min(A, 0) and log Q = max(A, 0) after every iteration, and one iteration adds a row term
// and a column term to A.  So A = K + f_i + g_j with K = tau_eff * importance: the whole Dykstra
// state of a block is K plus 2M potentials.  With kappa_ij = exp(K_ij - max_j K_ij) (the first row
// scaling makes a per-row factor of the start irrelevant) and the scalings U_i = exp(f_i), V_j = exp(g_j)
// one iteration is
//     e_ij = min(kappa_ij U_i V_j, 1);   R_i = N / sum_j e_ij;   C_j = N / sum_i e_ij R_i;
//     U_i *= R_i;   V_j *= C_j
// which is lines 3-6 of Algorithm 1 in exact arithmetic: the row scaling acts on the plan capped by
// the previous iteration, the column scaling on the row-scaled plan, and the cap with its dual is the
// min(., 1) at the top of the next pass (App. A.2 listing, same order of operations).  The kernel keeps
// kappa_ij U_i as one number per entry (updated by R_i every iteration), so an iteration costs four
// operations per entry - multiply-and-clamp, add, fused multiply-add, multiply - and no transcendental.
//
// Precision.  Default: everything in double (MI355X issues fp64 vector operations at 16 lanes/clk/SIMD),
// which reproduces a double-precision reference to ~1e-13.  FAST: the first kWarmIters iterations in
// double, then the loop in fp32 (a shorter instruction, and half the registers: three waves per SIMD
// instead of two) on kappa32 = fl32(kappa U V) with fp32 scalings relative to the double ones, which are
// kept as logarithms.  fp32 has 8 exponent bits, so every kChunk iterations the relative scalings are
// checked and, when one has drifted past 2^+-kDriftBits, their logarithms are added to the double ones and
// kappa32 is rebuilt as fl32(exp(K - row max + log U + log V)) from a fresh read of the importance (kappa
// itself is not kept: the kernel is budgeted the registers of three waves per SIMD).  Rebuilt entries are clamped to about
// [2^-120, 2^80]; within the drift bound (2^+-80 for a product of a row and a column scaling) a clamped
// entry is still >= 1 (capped) or <= 2^-40 (nothing).
//
// Layout.  A block is spread over LPB = GX*GY lanes as a GY x GX grid of TH x TW register tiles
// (TH = M/GY rows, TW = M/GX columns); a wave holds 64/LPB blocks.  Row sums are reduced across the GX
// lanes of a lane-row by recursive halving (reduce-scatter): after log2(GX) exchange steps every lane
// owns TH/GX complete row sums, computes their reciprocals once, and the results are gathered back the
// same way.  To keep every exchange a fixed set of registers (no selects), register a of lane gx holds
// tile row a ^ (gx << log2(TH/GX)); columns likewise over the GY lanes of a lane-column.
#pragma once
#include <type_traits>

#include "lanes.hpp"
#include "problem.hpp"
#include "rounding.hpp"

namespace tsenor_dev {

constexpr double kMinLogKernel = -700.0;  // exp(-700) is still a normal double
constexpr int kIdxBits = 12;              // flat index within a block: up to 64*64 entries
constexpr int kWarmIters = 4;             // FAST: iterations done in double before switching to fp32
constexpr int kRowChunks64 = 2;           // M = 64: the 8 x 8 tile is loaded in this many pieces (loads in flight cost registers)
constexpr int kChunk = 8;                 // FAST: iterations between range checks of the fp32 scalings
constexpr int kDriftBits = 40;            // FAST: fold the fp32 scalings back beyond 2^+-kDriftBits
constexpr double kLogFloor32 = -83.0;     // FAST: rebuilt entries are kept within [e^-83, e^55] ~ [2^-120, 2^80]
constexpr double kLogCeil32 = 55.0;


constexpr int ilog2(int x) { return x <= 1 ? 0 : 1 + ilog2(x / 2); }

// Per-M tiling.  XM[s] / YM[s]: lane masks of the exchange steps along a lane-row / lane-column.
// The top bit of XM[s] is lane bit NX-1-s (mirror masks keep the exchanges on DPP); YM[s] is a single
// lane bit, listed cheapest mechanism first because the first step moves the most registers.
// SMALL: a finer tiling (more lanes per block, fewer entries per lane) for launches that cannot fill the
// chip anyway: the dependent chain of an iteration is shorter.  Where a tile has fewer rows than the
// lane-row has lanes, the last exchange steps of a reduction have no registers left to split: they add the
// partner's value into the same register instead (both lanes end up owning the same sum).
template <int M, bool SMALL = false>
struct Tiling;
template <>
struct Tiling<4, false> {
  static constexpr int NX = 0, NY = 0;
  static constexpr int XM[1] = {1}, YM[1] = {1};
  static constexpr bool STORE_E = true;
};
template <>
struct Tiling<8, false> {
  static constexpr int NX = 1, NY = 1;
  static constexpr int XM[1] = {1}, YM[1] = {2};
  static constexpr bool STORE_E = true;
};
template <>
struct Tiling<16, false> {
  static constexpr int NX = 2, NY = 1;  // 8 lanes per block, 8 x 4 tiles
  static constexpr int XM[2] = {3, 1}, YM[1] = {4};
  static constexpr bool STORE_E = true;
};
template <>
struct Tiling<32, false> {
  static constexpr int NX = 3, NY = 2;  // 32 lanes per block, 8 x 4 tiles
  static constexpr int XM[3] = {7, 3, 1}, YM[2] = {8, 16};
  static constexpr bool STORE_E = true;
};
template <>
struct Tiling<64, false> {
  static constexpr int NX = 3, NY = 3;  // 64 lanes per block, 8 x 8 tiles; too large to hold e as doubles
  static constexpr int XM[3] = {7, 3, 1}, YM[3] = {8, 16, 32};
  static constexpr bool STORE_E = false;
};
template <>
struct Tiling<4, true> {
  static constexpr int NX = 1, NY = 1;  // 4 lanes per block, 2 x 2 tiles
  static constexpr int XM[1] = {1}, YM[1] = {2};
  static constexpr bool STORE_E = true;
};
template <>
struct Tiling<8, true> {
  static constexpr int NX = 2, NY = 2;  // 16 lanes per block, 2 x 2 tiles
  static constexpr int XM[2] = {3, 1}, YM[2] = {8, 4};
  static constexpr bool STORE_E = true;
};
template <>
struct Tiling<16, true> {
  static constexpr int NX = 2, NY = 2;  // 16 lanes per block, 4 x 4 tiles
  static constexpr int XM[2] = {3, 1}, YM[2] = {8, 4};
  static constexpr bool STORE_E = true;
};
template <>
struct Tiling<32, true> {
  static constexpr int NX = 3, NY = 3;  // 64 lanes per block, 4 x 4 tiles
  static constexpr int XM[3] = {7, 3, 1}, YM[3] = {8, 16, 32};
  static constexpr bool STORE_E = true;
};

// registers a lane owns after a reduce-scatter of `count` values over 2^steps lanes (at least one)
constexpr int owned(int count, int steps) { return (count >> steps) > 0 ? (count >> steps) : 1; }
// lane coordinate -> register offset of the row mapping: the top log2(TH) bits of gx if the tile has fewer
// rows than the lane-row has lanes, gx shifted up otherwise
constexpr int shift_lane(int x, int sh) { return sh >= 0 ? x << sh : x >> -sh; }

// 1/d from the hardware estimate x0.  A scaling factor is applied once and the sums of the next iteration see
// its error, so errors of the reciprocal do not accumulate over the iterations, while every refinement step sits
// in the dependent chain of each of them.  Double: x0 has ~24 bits; with e = 1 - d x0 one Newton step
// x0 (1 + e) leaves e^2 ~ 2^-48, two fused operations.  Float: the estimate itself (1 ulp).
__device__ __forceinline__ double fast_rcp(double d) {
  const double x = __builtin_amdgcn_rcp(d);
  return fma(fma(-d, x, 1.0), x, x);
}
__device__ __forceinline__ float fast_rcp(float d) { return __builtin_amdgcn_rcpf(d); }
__device__ __forceinline__ double clamp01(double x) { return fmin(fmax(x, 0.0), 1.0); }
__device__ __forceinline__ float clamp01(float x) { return fminf(fmaxf(x, 0.0f), 1.0f); }
__device__ __forceinline__ double vmax(double a, double b) { return fmax(a, b); }
__device__ __forceinline__ float vmax(float a, float b) { return fmaxf(a, b); }
__device__ __forceinline__ double vfma(double a, double b, double c) { return fma(a, b, c); }
__device__ __forceinline__ float vfma(float a, float b, float c) { return fmaf(a, b, c); }

// Recursive halving over the lanes of a lane-row.  v[0..TH): partial sums, register a <-> tile row
// a ^ shift_lane(gx, SH).  Afterwards v[0 .. owned(TH, NX)) hold complete sums.
template <class T, class real, int TH, int S = 0>
__device__ __forceinline__ void reduce_scatter_x(real (&v)[TH]) {
  if constexpr (S < T::NX) {
    constexpr int SH = ilog2(TH) - T::NX;
    constexpr int h = TH >> (S + 1);
    if constexpr (h >= 1) {
      constexpr int am = shift_lane(T::XM[S], SH) & (2 * h - 1);  // register index of the partner's matching value
#pragma unroll
      for (int a = 0; a < h; ++a) v[a] += lane_xor<T::XM[S]>(v[a ^ am]);
    } else {
      v[0] += lane_xor<T::XM[S]>(v[0]);  // no registers left to split: both lanes keep the sum
    }
    reduce_scatter_x<T, real, TH, S + 1>(v);
  }
}
template <class T, class real, int TH, int S = T::NX - 1>
__device__ __forceinline__ void all_gather_x(real (&v)[TH]) {
  if constexpr (S >= 0) {
    constexpr int SH = ilog2(TH) - T::NX;
    constexpr int h = TH >> (S + 1);
    if constexpr (h >= 1) {
      constexpr int am = shift_lane(T::XM[S], SH) & (2 * h - 1);
#pragma unroll
      for (int a = 0; a < h; ++a) v[a ^ am] = lane_xor<T::XM[S]>(v[a]);
    }
    all_gather_x<T, real, TH, S - 1>(v);
  }
}
// Maximum over the lanes of a lane-row of a value per tile row (all TH registers, butterfly): afterwards
// every lane holds the maximum of each of its tile rows.
template <class T, int TH, int S = 0>
__device__ __forceinline__ void all_reduce_max_x(float (&v)[TH]) {
  if constexpr (S < T::NX) {
    constexpr int SH = ilog2(TH) - T::NX;
    constexpr int am = shift_lane(T::XM[S], SH) & (TH - 1);
    float o[TH];
#pragma unroll
    for (int a = 0; a < TH; ++a) o[a] = lane_xor<T::XM[S]>(v[a ^ am]);
#pragma unroll
    for (int a = 0; a < TH; ++a) v[a] = fmaxf(v[a], o[a]);
    all_reduce_max_x<T, TH, S + 1>(v);
  }
}

// The same over the lanes of a lane-column; step s pairs lanes that differ in lane bit YM[s].
template <class T, class real, int TW, int S = 0>
__device__ __forceinline__ void reduce_scatter_y(real (&v)[TW]) {
  if constexpr (S < T::NY) {
    constexpr int h = TW >> (S + 1);
    if constexpr (h >= 1) {
#pragma unroll
      for (int b = 0; b < h; ++b) v[b] += lane_xor<T::YM[S]>(v[b + h]);
    } else {
      v[0] += lane_xor<T::YM[S]>(v[0]);
    }
    reduce_scatter_y<T, real, TW, S + 1>(v);
  }
}
// (steps S down to LAST; the default is the whole gather)
template <class T, class real, int TW, int S = T::NY - 1, int LAST = 0>
__device__ __forceinline__ void all_gather_y(real (&v)[TW]) {
  if constexpr (S >= LAST && S >= 0) {
    constexpr int h = TW >> (S + 1);
    if constexpr (h >= 1) {
#pragma unroll
      for (int b = 0; b < h; ++b) v[b + h] = lane_xor<T::YM[S]>(v[b]);
    }
    all_gather_y<T, real, TW, S - 1, LAST>(v);
  }
}
// the lowest step of all_gather_y whose move goes through the LDS crossbar (0: none does, or it is the last one)
template <class T, int TW, int S = 0>
constexpr int gather_split_y() {
  if constexpr (S < T::NY) {
    constexpr int m = T::YM[S];
    constexpr bool crossbar = m < 32 && m != 1 && m != 2 && m != 3 && m != 7 && m != 15 && m != 8;
    if constexpr (crossbar && (TW >> (S + 1)) >= 1)
      return S;
    else
      return gather_split_y<T, TW, S + 1>();
  } else {
    return 0;
  }
}
// register offset of a lane along y: lane bit YM[s] set <-> register bit log2(TW >> (s+1))
template <class T, int TW, int S = 0>
__device__ __forceinline__ int reg_xor_y(int q) {
  if constexpr (S < T::NY)
    return ((q & T::YM[S]) ? (TW >> (S + 1)) : 0) | reg_xor_y<T, TW, S + 1>(q);
  else
    return 0;
}

// An iteration alternates between two kinds of code: long runs of independent per-entry arithmetic, and the
// short dependent chains between them (exchange steps of a reduction, reciprocal, gather of the result) on
// which the next run waits.  A wave raises its priority for the chains, so that the SIMD issues their few
// instructions ahead of another wave's long run instead of behind it: with equal priorities the waves of a
// SIMD fell into step and stalled together (measured: 11-16 % of the fp32 loop, 1-2 % of the double one).
__device__ __forceinline__ void chain_phase(bool on) {
  if (on)
    __builtin_amdgcn_s_setprio(1);
  else
    __builtin_amdgcn_s_setprio(0);
}

// One iteration of Algorithm 1 (lines 3-6) on the register tile of this lane.  The row scalings are folded
// into the tile as they are found (kap holds kappa_ij U_i), so an entry costs one multiply with its column
// scaling, and only the scalings of the rows this lane owns are kept as numbers (Uown, for the potentials at
// the end).  `floor_` bounds the sums from below (keeps the scalings finite on degenerate input).  STORE
// keeps the capped entries of the row pass for the column pass; otherwise they are recomputed from an
// opaque copy of V (for tiles too large to hold twice: without the copy the compiler keeps the row pass's
// values alive and spills them).
// ADAPT (early exit): `frozen` lanes apply factors of exactly 1 (their block has stopped; its state no longer
// changes), and the largest |factor - 1| among the rows and columns this lane owns is returned.
template <class T, bool STORE, bool LDS_GATHER = false, bool ADAPT = false, class real, int TH, int TW, int OR>
__device__ __forceinline__ real dykstra_iteration(real (&kap)[TH][TW], real (&Uown)[OR], real (&V)[TW], real Nd,
                                                  real floor_, real* xr = nullptr, int rx = 0, bool frozen = false) {
  real worst = 0;
  constexpr int OWN_R = owned(TH, T::NX), OWN_C = owned(TW, T::NY);
  static_assert(OR == OWN_R, "one scaling per owned row");
  real e[STORE ? TH : 1][STORE ? TW : 1];
  real R[TH], C[TW];
  // projection onto C1 (line 3) of the plan capped by the previous iteration
#pragma unroll
  for (int a = 0; a < TH; ++a) {
    real s = 0;
#pragma unroll
    for (int b = 0; b < TW; ++b) {
      const real ev = clamp01(kap[a][b] * V[b]);
      if constexpr (STORE) e[a][b] = ev;
      s = b == 0 ? ev : s + ev;  // (0 + x is not a no-op for the compiler: it would keep the add)
    }
    R[a] = s;
  }
  chain_phase(true);
  reduce_scatter_x<T, real, TH>(R);
#pragma unroll
  for (int a = 0; a < OWN_R; ++a) {
    R[a] = Nd * fast_rcp(vmax(R[a], floor_));
    if constexpr (ADAPT) {
      worst = vmax(worst, fabs(R[a] - real(1)));
      R[a] = frozen ? real(1) : R[a];
    }
    Uown[a] *= R[a];
  }
  if constexpr (LDS_GATHER) {
    // the owner of a row leaves its scaling in LDS and every lane of the lane-row picks up all TH of them:
    // LDS instructions instead of vector-ALU moves.  The lanes of a wave run in lock step, so the exchange
    // needs no barrier, only that the compiler keeps the accesses where they are.
#pragma unroll
    for (int a = 0; a < OWN_R; ++a) xr[a ^ rx] = R[a];
    asm volatile("" ::: "memory");
#pragma unroll
    for (int a = OWN_R; a < TH; ++a) R[a] = xr[a ^ rx];  // (the owned rows' factors are at hand)
    asm volatile("" ::: "memory");
  } else {
    all_gather_x<T, real, TH>(R);
  }
  chain_phase(false);
  // projection onto C2 (line 4)
  real Vc[TW];
#pragma unroll
  for (int b = 0; b < TW; ++b) {
    Vc[b] = V[b];
    if constexpr (!STORE) asm volatile("" : "+v"(Vc[b]));
  }
#pragma unroll
  for (int b = 0; b < TW; ++b) {
    real s = 0;
#pragma unroll
    for (int a = 0; a < TH; ++a) {
      real ev;
      if constexpr (STORE)
        ev = e[a][b];
      else
        ev = clamp01(kap[a][b] * Vc[b]);
      s = vfma(ev, R[a], s);
    }
    C[b] = s;
  }
  chain_phase(true);
  reduce_scatter_y<T, real, TW>(C);
#pragma unroll
  for (int b = 0; b < OWN_C; ++b) {
    C[b] = Nd * fast_rcp(vmax(C[b], floor_));
    if constexpr (ADAPT) {
      worst = vmax(worst, fabs(C[b] - real(1)));
      C[b] = frozen ? real(1) : C[b];
    }
  }
  // the owner of a column applies its factor and the new scalings (not the factors) are gathered: every lane
  // would have formed the same products
#pragma unroll
  for (int b = 0; b < OWN_C; ++b) V[b] *= C[b];
  // the steps of the gather down to the last one that goes through the LDS crossbar are issued before the
  // rescaling of the tile, the rest after it: the tile's multiplies cover the latency of those moves
  constexpr int SPLIT = gather_split_y<T, TW>();
  all_gather_y<T, real, TW, T::NY - 1, SPLIT>(V);
  chain_phase(false);
  if constexpr (SPLIT > 0) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int a = 0; a < TH; ++a)
#pragma unroll
    for (int b = 0; b < TW; ++b) kap[a][b] *= R[a];
  if constexpr (SPLIT > 0) {
    __builtin_amdgcn_sched_barrier(0);
    all_gather_y<T, real, TW, SPLIT - 1>(V);
  }
  // lines 5-6 (cap and dual update) are the clamp at the top of the next pass
  return worst;
}

// x * y with the result clamped to [0, 1] by the output modifier: one instruction at the full fp32 rate
// (measured on MI355X: 1.2 ns per wave-instruction per SIMD, as a plain v_mul_f32; v_min_f32 / v_max_f32 /
// v_med3_f32 take 1.9 ns).  Written as the bare instruction so that it stays this one.
__device__ __forceinline__ float mul_clamp01(float x, float y) {
  float r;
  asm("v_mul_f32_e64 %0, %1, %2 clamp" : "=v"(r) : "v"(x), "v"(y));
  return r;
}

// max(a, b) as the bare instruction: fmaxf() first quiets a possible signalling NaN in an operand the compiler
// has not just computed (the loop-invariant floor below), one more instruction in every iteration
__device__ __forceinline__ float max_as_is(float a, float b) {
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}

// The same iteration in single precision.  kap stays as rebuilt (no rounding accumulates in it); the scalings
// U (every tile row) and V (every tile column) are kept as numbers, and the capped entry is
//     e_ij = clamp(kap_ij * (U_i V_j)):  a multiply, a multiply with the clamp modifier, the add of the row
// sum and the multiply-add of the column sum per entry, all at the full fp32 rate.  A scaling grows by at most
// 2^10 per iteration (keeps everything finite on degenerate input).
// ADAPT as in dykstra_iteration.
template <class T, bool LDS_GATHER = false, bool ADAPT = false, int TH, int TW>
__device__ __forceinline__ float dykstra_iteration_f32(const float (&kap)[TH][TW], float (&U)[TH], float (&V)[TW],
                                                       float Nf, float2* xr = nullptr, int rx = 0,
                                                       bool frozen = false) {
  constexpr int OWN_R = owned(TH, T::NX), OWN_C = owned(TW, T::NY);
  float worst = 0;
  float e[TH][TW], R[TH], C[TW];
#pragma unroll
  for (int a = 0; a < TH; ++a) {
#pragma unroll
    for (int b = 0; b < TW; ++b) {
      e[a][b] = mul_clamp01(kap[a][b], U[a] * V[b]);
      R[a] = b == 0 ? e[a][b] : R[a] + e[a][b];
    }
  }
  chain_phase(true);
  reduce_scatter_x<T, float, TH>(R);
#pragma unroll
  for (int a = 0; a < OWN_R; ++a) {
    R[a] = fminf(Nf * fast_rcp(R[a]), 1024.0f);  // factor of an owned row (a NaN from an empty row gives the cap)
    if constexpr (ADAPT) {
      worst = fmaxf(worst, fabsf(R[a] - 1.0f));
      R[a] = frozen ? 1.0f : R[a];
    }
  }
  if constexpr (LDS_GATHER) {
    // the owner of a row updates its scaling and leaves factor and scaling in LDS; the other lanes of the
    // lane-row pick both up in one 8-byte read per row instead of multiplying each scaling themselves
#pragma unroll
    for (int a = 0; a < OWN_R; ++a) {
      U[a] *= R[a];
      xr[a ^ rx] = make_float2(R[a], U[a]);
    }
    asm volatile("" ::: "memory");
#pragma unroll
    for (int a = OWN_R; a < TH; ++a) {
      const float2 ru = xr[a ^ rx];
      R[a] = ru.x;
      U[a] = ru.y;
    }
    asm volatile("" ::: "memory");
  } else {
    all_gather_x<T, float, TH>(R);
#pragma unroll
    for (int a = 0; a < TH; ++a) U[a] *= R[a];
  }
  chain_phase(false);
#pragma unroll
  for (int b = 0; b < TW; ++b) {
#pragma unroll
    for (int a = 0; a < TH; ++a) C[b] = a == 0 ? e[a][b] * R[a] : fmaf(e[a][b], R[a], C[b]);
  }
  chain_phase(true);
  reduce_scatter_y<T, float, TW>(C);
#pragma unroll
  for (int b = 0; b < OWN_C; ++b) {
    C[b] = Nf * fast_rcp(max_as_is(C[b], Nf * 0x1p-10f));
    if constexpr (ADAPT) {
      worst = fmaxf(worst, fabsf(C[b] - 1.0f));
      C[b] = frozen ? 1.0f : C[b];
    }
  }
#pragma unroll
  for (int b = 0; b < OWN_C; ++b) V[b] *= C[b];
  all_gather_y<T, float, TW>(V);
  chain_phase(false);
  return worst;
}

__device__ __forceinline__ void compare_exchange(double& lo, double& hi) {
  const double a = fmin(lo, hi), b = fmax(lo, hi);
  lo = a;
  hi = b;
}

// min(a, -b) as one instruction (fmin() would first quiet possible signalling NaNs in operands the compiler
// has not computed itself, one more instruction each)
__device__ __forceinline__ double min_with_negated(double a, double b) {
  double r;
  asm("v_min_f64 %0, %1, -%2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}

// Sign convention of the keys between sort stages: the lanes whose bit SB is set hold their keys negated
// (SB = 0: nobody).  Moves from convention SB to convention B: one xor per key in the lanes that change.
template <int SB, int B, int E>
__device__ __forceinline__ void sort_resign(double (&c)[E], int q) {
  if constexpr (SB != B) {
    const bool flip = ((q & SB) != 0) != ((q & B) != 0);
    const int mask = flip ? (int)0x80000000 : 0;
#pragma unroll
    for (int r = 0; r < E; ++r) c[r] = __hiloint2double(__double2hiint(c[r]) ^ mask, __double2loint(c[r]));
  }
}

// Ascending bitonic sort of E*LPB distinct positive doubles spread over LPB lanes (position q*E + r).
// Every merge starts with the mirrored compare (position p against p ^ (k-1)), after which the smaller
// key always belongs at the lower position, so no direction flags are needed.
// A stage across lanes: the lane whose bit is clear keeps the smaller of its key and the partner's, the other
// lane the larger.  With the keys of the second kind of lane held negated, both are min(own, -partner's):
// two cross-lane moves and one instruction per key instead of a compare and two selects (the selects and the
// moves issue at the double-precision rate on this chip), plus one xor per key where the convention changes.
template <int E, int LPB, int J, int SB = 0>
__device__ __forceinline__ void sort_half_cleaners(double (&c)[E], int q) {
  if constexpr (J >= 1) {
    if constexpr (J < E) {
      sort_resign<SB, 0>(c, q);
#pragma unroll
      for (int r = 0; r < E; ++r) {
        const int pr = r ^ J;
        if (pr > r) compare_exchange(c[r], c[pr]);
      }
      sort_half_cleaners<E, LPB, J / 2, 0>(c, q);
    } else {
      constexpr int lm = J / E;
      sort_resign<SB, lm>(c, q);
#pragma unroll
      for (int r = 0; r < E; ++r) c[r] = min_with_negated(c[r], lane_xor<lm>(c[r]));
      // with 64 keys per lane the scheduler otherwise starts the next stage's exchanges early and spills them
      if constexpr (E >= 64) __builtin_amdgcn_sched_barrier(0);
      sort_half_cleaners<E, LPB, J / 2, lm>(c, q);
    }
  } else {
    sort_resign<SB, 0>(c, q);
  }
}

template <int E, int LPB, int K = 2>
__device__ __forceinline__ void sort_ascending(double (&c)[E], int q) {
  if constexpr (K <= E * LPB) {
    if constexpr (K <= E) {
#pragma unroll
      for (int r = 0; r < E; ++r) {
        const int pr = r ^ (K - 1);
        if (pr > r) compare_exchange(c[r], c[pr]);
      }
      sort_half_cleaners<E, LPB, K / 4, 0>(c, q);
    } else {
      constexpr int lm = K / E - 1, bit = K / E / 2;
      sort_resign<0, bit>(c, q);
      // position r meets the partner lane's position E-1-r; two registers at a time keeps this in place
#pragma unroll
      for (int r = 0; r < E / 2; ++r) {
        const double o_lo = lane_xor<lm>(c[E - 1 - r]), o_hi = lane_xor<lm>(c[r]);
        c[r] = min_with_negated(c[r], o_lo);
        c[E - 1 - r] = min_with_negated(c[E - 1 - r], o_hi);
      }
      if constexpr (E >= 64) __builtin_amdgcn_sched_barrier(0);
      sort_half_cleaners<E, LPB, K / 4, bit>(c, q);
    }
    sort_ascending<E, LPB, K * 2>(c, q);
  }
}

// calls f(integral_constant<A0>) for A0 = 0, NA, 2 NA, ... < TH: a tile is loaded NA rows at a time
template <int A0, int NA, int TH, class F>
__device__ __forceinline__ void row_chunks(F& f) {
  if constexpr (A0 < TH) {
    f(std::integral_constant<int, A0>{});
    row_chunks<A0 + NA, NA, TH>(f);
  }
}

template <int M, bool FAST, bool ADAPT = false, bool SMALL = false>
struct DykstraLaunch {
  // with the early exit the waves of a launch run for very different times; one-wave workgroups let the
  // dispatcher refill every wave slot as it frees (a four-wave workgroup holds its slots until its slowest wave).
  // The small tiles carry the rounding behind the iterations, whose steps synchronise one wave at a time.
  static constexpr int kWavesPerGroup = (ADAPT || SMALL) ? 1 : 4;
  static constexpr int kThreads = kWavesPerGroup * kWave;
  // waves per SIMD the register budget is set for.  The fp32 loop wants more than two (one wave issues at
  // most every ~5 cycles, an fp32 instruction occupies the SIMD for 2-3): three waves of 168 registers.  For
  // M <= 32 the whole kernel fits them without spills (four waves, 128 registers and a few spills outside the
  // loop, measured the same).  For M = 64 the loop fits (64 + 64 registers for the tile and the capped entries)
  // but the double-precision phases around it do not (the warm-up iterations on a tile of 64 doubles, the sort
  // of 64 keys): they spill ~90 registers to scratch, none inside the loop, and the kernel is 5.5 % faster than
  // with two waves (not with the early exit, where a block may run a dozen iterations and the code around the loop
  // is most of the work: two waves there).  The double-precision loop holds twice the state: two waves of up to
  // 256 registers.
  static constexpr int kWavesPerSimd = FAST && !(M == 64 && ADAPT) ? 3 : 2;
};

// ZERO_T: the instantiation for T = 0 (no iterations, keys are K itself).  It is a template parameter
// rather than a branch because keeping both paths in one kernel costs the iterating path ~40 registers.
// SMALL: the finer tiling, for launches that cannot fill the chip.  There the whole path stays in this kernel:
// a block lives in one wave from its tile load to its mask, so the sorted scan order goes to LDS instead of the
// workspace and Algorithm 2 (greedy selection with M lanes per block, local search, mask write) runs behind the
// sort; no further kernel follows.
template <int M, bool FAST, bool ZERO_T = false, bool SMALL = false, bool ADAPT = false>
__global__ __launch_bounds__((DykstraLaunch<M, FAST, ADAPT, SMALL>::kThreads), (DykstraLaunch<M, FAST, ADAPT, SMALL>::kWavesPerSimd)) void dykstra_sort_kernel(
    Batch batch) {
  using T = Tiling<M, SMALL>;
  const int which = find_problem(batch, blockIdx.x);
  const DevProblem p = batch.e[which].p;
  unsigned short* order = batch.e[which].order;
  double* plan_out = batch.e[which].plan_out;
  double* tau_eff_out = batch.e[which].tau_eff_out;
  const unsigned int group = blockIdx.x - batch.first[which];  // workgroup index within the matrix
  constexpr int GX = 1 << T::NX, GY = 1 << T::NY, TH = M / GY, TW = M / GX, LPB = GX * GY, BPW = kWave / LPB,
                E = TH * TW, SHX = ilog2(TH) - T::NX, WPG = DykstraLaunch<M, FAST, ADAPT, SMALL>::kWavesPerGroup;
  const int lane = threadIdx.x & (kWave - 1), wave_in_group = threadIdx.x / kWave;
  const int64_t wave = (int64_t)group * WPG + wave_in_group;
  const int q = lane % LPB, gx = q % GX, gy = q / GX;
  int64_t blk = wave * BPW + lane / LPB;
  const bool active = blk < p.nblocks;
  if (!active) blk = p.nblocks - 1;  // idle lanes shadow the last block and write nothing
  const int64_t r0 = (blk / p.bc) * M, c0 = (blk % p.bc) * M;
  const double tau_eff = tau_eff_of(batch.e[which]);
  if (tau_eff_out && group == 0 && threadIdx.x == 0) *tau_eff_out = tau_eff;

  // register (a, b) of this lane <-> in-kernel coordinates (ri, cj) of the block.  Each phase of the
  // kernel takes its own opaque copy of the lane offsets, so that element addresses are recomputed where
  // they are needed instead of being kept in registers across the iteration loop.
  const int rx = shift_lane(gx, SHX), ry = reg_xor_y<T, TW>(q);
  auto fresh = [](int v) {
    asm volatile("" : "+v"(v));
    return v;
  };
  // with `transpose` the in-kernel rows are the matrix columns, which turns "rows first" into
  // "columns first" (TSENOR_FLAG_COLS_FIRST)
  auto mat_row = [&](int ri, int cj) { return p.transpose ? cj : ri; };
  auto mat_col = [&](int ri, int cj) { return p.transpose ? ri : cj; };

  // tile addressing of one phase, from that phase's copy of the lane offsets
  auto addr_of = [&](int rxp, int ryp) {
    int ri[TH], cj[TW];
#pragma unroll
    for (int a = 0; a < TH; ++a) ri[a] = gy * TH + (a ^ rxp);
#pragma unroll
    for (int b = 0; b < TW; ++b) cj[b] = gx * TW + (b ^ ryp);
    return tile_addr<TH, TW>(p, r0, c0, ri, cj);
  };
  // rows of a tile loaded at a time: the fp32 variant lives in half the registers (two halves); the 8 x 8
  // tiles of M = 64 would keep 64 loads with their addresses in flight and spill
  constexpr int NA = M == 64 ? TH / kRowChunks64 : (FAST && TH >= 8) ? TH / 2 : TH;

  double c[E];  // sort keys
  int iters_done = 0;
  double kap[ZERO_T ? 1 : TH][ZERO_T ? 1 : TW];
  // Normaliser of every in-kernel row: kappa = exp(K - mrow) <= ~1.  Any per-row constant gives the same
  // iterates, because the first step of Algorithm 1 rescales every row (with TSENOR_FLAG_COLS_FIRST: every
  // column, which is the in-kernel row); a single precision value a little above the row's largest K is
  // enough.  Per row rather than per block, so that one huge entry does not push the other rows of its
  // block below the range of a double.
  float mrow[TH];
  {
    const int rx0 = fresh(rx), ry0 = fresh(ry);
    const auto addr = addr_of(rx0, ry0);
    // the plan (a diagnostic output) in a pass of its own, before the keys exist and with its own loads: an
    // exp() inside the key pass, or keys kept alive across it, costs registers (spills for M = 64)
    if constexpr (ZERO_T) {
      if (plan_out && active) {
        auto plan_rows = [&](auto first) {
          constexpr int A0 = decltype(first)::value;
          float imp[NA][TW];
          tile_importance<A0, NA>(p, addr, imp);
#pragma unroll
          for (int a = 0; a < NA; ++a)
#pragma unroll
            for (int b = 0; b < TW; ++b) {
              const int ri = gy * TH + ((A0 + a) ^ rx0), cj = gx * TW + (b ^ ry0);
              plan_out[(r0 + mat_row(ri, cj)) * p.cols + c0 + mat_col(ri, cj)] = exp(tau_eff * (double)imp[a][b]);
              __builtin_amdgcn_sched_barrier(0);
            }
        };
        row_chunks<0, NA, TH>(plan_rows);
      }
    }
    auto rows = [&](auto first) {
      constexpr int A0 = decltype(first)::value;
      float imp[NA][TW];
      tile_importance<A0, NA>(p, addr, imp);
#pragma unroll
      for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int b = 0; b < TW; ++b) {
          const double K = tau_eff * (double)imp[a][b];  // K of Algorithm 1 line 1
          if constexpr (ZERO_T) {
            // no iterations: the greedy order is descending K itself.  Bit patterns of non-negative doubles
            // order like the doubles: pattern(2^1023) - pattern(K) reverses the order for every finite
            // K >= 0 and is again the pattern of a positive double
            const int ri = gy * TH + ((A0 + a) ^ rx0), cj = gx * TW + (b ^ ry0);
            const unsigned long long idx = (unsigned long long)(mat_row(ri, cj) * M + mat_col(ri, cj));
            const unsigned long long bits = (unsigned long long)__double_as_longlong(K);
            const unsigned long long key = (0x7FE0000000000000ull - bits) & ~((1ull << kIdxBits) - 1);
            c[(A0 + a) * TW + b] = __longlong_as_double((long long)(key | idx));
          } else {
            kap[A0 + a][b] = K;
            const float up = __double2float_ru(K);
            mrow[A0 + a] = b == 0 ? up : fmaxf(mrow[A0 + a], up);
          }
        }
    };
    row_chunks<0, NA, TH>(rows);
  }
  if constexpr (!ZERO_T) {
    all_reduce_max_x<T, TH>(mrow);
#pragma unroll
    for (int a = 0; a < TH; ++a)
#pragma unroll
      for (int b = 0; b < TW; ++b) {
        kap[a][b] = exp(fmax(kap[a][b] - (double)mrow[a], kMinLogKernel));
        __builtin_amdgcn_sched_barrier(0);  // one exp at a time: interleaving them only costs registers
      }

    const double Nd = (double)p.N;
    iters_done = p.T;
    const long long cycles0 = clock64(), ticks0 = wall_clock64();
    // logs of the scalings of the rows and columns this lane owns (the first registers after a
    // reduce-scatter); the other lanes of the lane-row / lane-column hold the same values for theirs
    constexpr int OWN_R = owned(TH, T::NX), OWN_C = owned(TW, T::NY);
    double lu_own[OWN_R], lv_own[OWN_C];
    // early exit: a block whose factors have passed the tolerance is frozen at that iteration
    bool frozen = false;
    auto freeze_if = [&](bool passed, int t_done) {
      if (!frozen && passed) {
        frozen = true;
        iters_done = t_done;
      }
    };
    // FAST: the tile of the fp32 phase, fl32(kap U V)
    float kap32[FAST ? TH : 1][FAST ? TW : 1];
    {
      double Uown[OWN_R], V[TW];
#pragma unroll
      for (int a = 0; a < OWN_R; ++a) Uown[a] = 1.0;
#pragma unroll
      for (int b = 0; b < TW; ++b) V[b] = 1.0;
      if constexpr (FAST) {
        // the entries are recomputed in the column pass: this phase must fit the registers of the fp32 loop
        const int t_double = p.T < kWarmIters ? p.T : kWarmIters;
        for (int t = 0; t < t_double; ++t) {
          double worst = dykstra_iteration<T, false, false, ADAPT>(kap, Uown, V, Nd, 1e-300, (double*)nullptr, 0, frozen);
          if constexpr (ADAPT) {
            if ((t + 1) % TSENOR_ADAPTIVE_CHECK_EVERY == 0) freeze_if(block_max<LPB>(worst) <= p.tol, t + 1);
          }
        }
      } else {
        // In the 32- and 64-wide kernels the row scalings of an iteration are gathered through LDS (measured
        // ~1 % faster than DPP moves; doing the same for the column scalings as well exposed a second LDS round
        // trip and gained nothing): lane-row r of the wave keeps its 8 row scalings at xrows[wave][r][0..8)
        constexpr bool kLdsGather = M >= 32 && !SMALL;
        __shared__ double xrows[kLdsGather ? WPG : 1][kLdsGather ? kWave >> T::NX : 1][TH];
        double* xr = kLdsGather ? &xrows[wave_in_group][lane >> T::NX][0] : nullptr;
        if constexpr (ADAPT) {
          // iteration count as a bound: every TSENOR_ADAPTIVE_CHECK_EVERY-th iteration the largest |factor - 1|
          // of the block is compared with the tolerance; a block that passes is frozen, the wave leaves when
          // all its blocks are
          for (int t = 0; t < p.T; ++t) {
            double worst =
                dykstra_iteration<T, T::STORE_E, kLdsGather, true>(kap, Uown, V, Nd, 1e-300, xr, rx, frozen);
            if ((t + 1) % TSENOR_ADAPTIVE_CHECK_EVERY == 0) {
              freeze_if(block_max<LPB>(worst) <= p.tol, t + 1);
              if (__all(frozen)) break;
            }
          }
        } else {
          for (int t = 0; t < p.T; ++t) dykstra_iteration<T, T::STORE_E, kLdsGather>(kap, Uown, V, Nd, 1e-300, xr, rx);
        }
      }
      if constexpr (FAST) {
        // The first tile of the fp32 phase comes from the double-precision tile while it is still at hand (it
        // holds kap U; a multiply with V and a conversion per entry, clamped like a rebuilt entry); only a later
        // rebuild has to read the importance again and go through exp().
        const double floor32 = 0x1.31c5957a47de2p-120, ceil32 = 0x1.45e3076d61699p+79;  // e^kLogFloor32, e^kLogCeil32
#pragma unroll
        for (int a = 0; a < TH; ++a)
#pragma unroll
          for (int b = 0; b < TW; ++b) kap32[a][b] = (float)fmin(fmax(kap[a][b] * V[b], floor32), ceil32);
      }
#pragma unroll
      for (int a = 0; a < OWN_R; ++a) {
        lu_own[a] = log(Uown[a]);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int b = 0; b < OWN_C; ++b) {
        lv_own[b] = log(V[b]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }

    if constexpr (FAST) {
      if (p.T > kWarmIters && !(ADAPT && __all(frozen))) {
        // fp32 phase: kap32 = fl32(kap U V) for the double scalings U V reached so far, and fp32 scalings
        // U32, V32 relative to them.  kap is not kept: a rebuild reloads the importance.
        float U32[TH], V32[TW];
        const float Nf = (float)p.N;
        const float hi = __builtin_ldexpf(1.0f, kDriftBits), lo = __builtin_ldexpf(1.0f, -kDriftBits);
        auto rebuild = [&]() {
          const int rx1 = fresh(rx), ry1 = fresh(ry);
          double lu[TH], lv[TW];
#pragma unroll
          for (int a = 0; a < OWN_R; ++a) lu[a] = lu_own[a];
#pragma unroll
          for (int b = 0; b < OWN_C; ++b) lv[b] = lv_own[b];
          all_gather_x<T, double, TH>(lu);
          all_gather_y<T, double, TW>(lv);
          const auto addr = addr_of(rx1, ry1);
          auto rows = [&](auto first) {
            constexpr int A0 = decltype(first)::value;
            float imp[NA][TW];
            tile_importance<A0, NA>(p, addr, imp);
#pragma unroll
            for (int a = 0; a < NA; ++a)
#pragma unroll
              for (int b = 0; b < TW; ++b) {
                const double K = tau_eff * (double)imp[a][b];
                const double full = (K - (double)mrow[A0 + a]) + (lu[A0 + a] + lv[b]);
                kap32[A0 + a][b] = (float)exp(fmin(fmax(full, kLogFloor32), kLogCeil32));
                __builtin_amdgcn_sched_barrier(0);
              }
          };
          row_chunks<0, NA, TH>(rows);
#pragma unroll
          for (int a = 0; a < TH; ++a) U32[a] = 1.0f;
#pragma unroll
          for (int b = 0; b < TW; ++b) V32[b] = 1.0f;
        };
        auto fold = [&]() {
#pragma unroll
          for (int a = 0; a < OWN_R; ++a) {
            lu_own[a] += log((double)U32[a]);
            __builtin_amdgcn_sched_barrier(0);
          }
#pragma unroll
          for (int b = 0; b < OWN_C; ++b) {
            lv_own[b] += log((double)V32[b]);
            __builtin_amdgcn_sched_barrier(0);
          }
        };
#pragma unroll
        for (int a = 0; a < TH; ++a) U32[a] = 1.0f;
#pragma unroll
        for (int b = 0; b < TW; ++b) V32[b] = 1.0f;
        bool all_frozen = false;
        for (int t = kWarmIters; t < p.T && !all_frozen;) {
          const int stop = (p.T - t > kChunk) ? t + kChunk : p.T;
          // (in fp32 the exchange also carries the updated scalings, which pays wherever a block spans lanes:
          // -6 % for M = 8, -10 % for M = 16; in double the 16-wide kernel is 1.5 % faster with DPP moves)
          constexpr bool kLdsGather32 = M >= 8;
          __shared__ float2 xrows32[kLdsGather32 ? WPG : 1][kLdsGather32 ? kWave >> T::NX : 1][TH];
          float2* xr = kLdsGather32 ? &xrows32[wave_in_group][lane >> T::NX][0] : nullptr;
          if constexpr (ADAPT) {
            for (; t < stop && !all_frozen; ++t) {
              const float worst =
                  dykstra_iteration_f32<T, kLdsGather32, true>(kap32, U32, V32, Nf, xr, rx, frozen);
              if ((t + 1) % TSENOR_ADAPTIVE_CHECK_EVERY == 0) {
                freeze_if(block_max<LPB>((double)worst) <= p.tol, t + 1);
                all_frozen = __all(frozen);
              }
            }
          } else {
            for (; t < stop; ++t) dykstra_iteration_f32<T, kLdsGather32>(kap32, U32, V32, Nf, xr, rx);
          }
          // (the scalings of the rows and columns this lane owns: every row and column has its owner, and the
          // other copies of a scaling are the same number)
          float mxs = U32[0], mns = U32[0];
#pragma unroll
          for (int a = 1; a < OWN_R; ++a) mxs = fmaxf(mxs, U32[a]), mns = fminf(mns, U32[a]);
#pragma unroll
          for (int b = 0; b < OWN_C; ++b) mxs = fmaxf(mxs, V32[b]), mns = fminf(mns, V32[b]);
          // wave-uniform: fold the fp32 scalings into the double ones when any lane's have drifted
          if (t < p.T && __any(!(mxs < hi && mns > lo))) {
            fold();
            rebuild();
          }
        }
        fold();
      }
    }

    if (group == 0 && threadIdx.x == 0) {
      WsHeader* h = batch.e[which].hdr;
      h->loop_cycles = (unsigned long long)(clock64() - cycles0);
      h->loop_ticks = (unsigned long long)(wall_clock64() - ticks0);
    }

    const int rx2 = fresh(rx), ry2 = fresh(ry);
    double lu[TH], lv[TW];
#pragma unroll
    for (int a = 0; a < OWN_R; ++a) lu[a] = lu_own[a];
#pragma unroll
    for (int b = 0; b < OWN_C; ++b) lv[b] = lv_own[b];
    all_gather_x<T, double, TH>(lu);
    all_gather_y<T, double, TW>(lv);
    const auto addr = addr_of(rx2, ry2);
    // log S^(T) = min(K + f_i + g_j, 0)
    // (K is not floored here as it is for kappa: entries too small for the iterations to see keep
    // their own order in the scan)
    auto log_plan = [&](float importance, int a, int b) {
      const double K = tau_eff * (double)importance;
      return fmin((K - (double)mrow[a]) + (lu[a] + lv[b]), 0.0);
    };
    // the plan (a diagnostic output) in a pass of its own, with its own loads: an exp() inside the key pass
    // costs it registers (spills for M = 64)
    if (plan_out && active) {
      auto plan_rows = [&](auto first) {
        constexpr int A0 = decltype(first)::value;
        float imp[NA][TW];
        tile_importance<A0, NA>(p, addr, imp);
#pragma unroll
        for (int a = 0; a < NA; ++a)
#pragma unroll
          for (int b = 0; b < TW; ++b) {
            const int ri = gy * TH + ((A0 + a) ^ rx2), cj = gx * TW + (b ^ ry2);
            plan_out[(r0 + mat_row(ri, cj)) * p.cols + c0 + mat_col(ri, cj)] = exp(log_plan(imp[a][b], A0 + a, b));
            __builtin_amdgcn_sched_barrier(0);
          }
      };
      row_chunks<0, NA, TH>(plan_rows);
    }
    auto rows = [&](auto first) {
      constexpr int A0 = decltype(first)::value;
      float imp[NA][TW];
      tile_importance<A0, NA>(p, addr, imp);
#pragma unroll
      for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int b = 0; b < TW; ++b) {
          const int ri = gy * TH + ((A0 + a) ^ rx2), cj = gx * TW + (b ^ ry2);
          const double key = log_plan(imp[a][b], A0 + a, b);
          const unsigned long long idx = (unsigned long long)(mat_row(ri, cj) * M + mat_col(ri, cj));
          const unsigned long long bits = (unsigned long long)__double_as_longlong(fabs(key));
          // descending key, ties by ascending flat index; + 2^52 keeps the pattern a normal double
          c[(A0 + a) * TW + b] =
              __longlong_as_double((long long)(((bits & ~((1ull << kIdxBits) - 1)) | idx) + (1ull << 52)));
        }
    };
    row_chunks<0, NA, TH>(rows);
  }

  sort_ascending<E, LPB>(c, q);
  // The stores below sit under `active`, and only the index bits of a key are stored: the compiler would move
  // the last stage's selects into that branch but has to leave its cross-lane moves outside, all of them
  // alive at once (spills for M = 64).  Using the keys here keeps every select next to its moves.
#pragma unroll
  for (int r = 0; r < E; ++r) asm volatile("" : "+v"(c[r]));

  if (active && q == 0 && batch.e[which].iters_done_out) batch.e[which].iters_done_out[blk] = iters_done;
  if constexpr (SMALL) {
    // Algorithm 2 behind the sort, in the same wave: the scan order of the wave's blocks through LDS
    static_assert(WPG == 1, "the rounding steps synchronise single-wave workgroups");
    __shared__ unsigned short scan[BPW][M * M];
    __shared__ RoundingLds<M, BPW> lds;
    unsigned short* mine = &scan[lane / LPB][0];
#pragma unroll
    for (int r = 0; r < E; ++r)
      mine[q * E + r] = (unsigned short)((unsigned long long)__double_as_longlong(c[r]) & ((1ull << kIdxBits) - 1));
    __syncthreads();
    const int placed = greedy_wide_scan<M, LPB>([&](int pos) { return (unsigned int)mine[pos]; }, p.N, lane, lds);
    if (batch.e[which].stats_out) {
      int missing = (active && q == 0) ? p.N * M - placed : 0;
      for (int s = 1; s < kWave; s <<= 1) missing += __shfl_xor(missing, s, kWave);
      if (lane == 0 && missing) atomicAdd(&batch.e[which].hdr->stats[0], (unsigned long long)missing);
    }
    local_search_and_write<M, LPB>(p, batch.e[which], blk, active, lane, lds);
  } else if (active) {
    unsigned short* dst = order + blk * (int64_t)(M * M) + q * E;
#pragma unroll
    for (int r = 0; r < E; ++r)
      dst[r] = (unsigned short)((unsigned long long)__double_as_longlong(c[r]) & ((1ull << kIdxBits) - 1));
  }
}

}  // namespace tsenor_dev
