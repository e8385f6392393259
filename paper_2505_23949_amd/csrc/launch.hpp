// Interface between the host code of the library and the kernels that depend on the block size M.  The
// kernels of every M are compiled in a translation unit of their own (launch_m4.hip ... launch_m64.hip, all of
// them instantiating launch_impl.hpp), so that the library builds in parallel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "problem.hpp"

namespace tsenor_dev {

// kernel variant of a problem: problems with the same variant can share one fused launch
struct Variant {
  int M;
  bool fast, zero_t;
  uint32_t greedy;  // 0: chosen by size, else the TSENOR_FLAG_GREEDY_* asked for
  bool small;       // the Dykstra kernel's small tiles (decided per problem, so that fusing never changes results)
  bool simple;      // TSENOR_FLAG_SIMPLE_ROUNDING
  bool adaptive;    // tol > 0: the early-exit instantiation of the Dykstra kernel
  bool operator==(const Variant& o) const {
    return M == o.M && fast == o.fast && zero_t == o.zero_t && greedy == o.greedy && small == o.small &&
           simple == o.simple && adaptive == o.adaptive;
  }
};

// Below this many blocks in a matrix the whole path runs in the one kernel with the small tiles (M <= 32, double
// iterations): with few waves a SIMD holds one or two, whose iteration time is the dependent chain, and the
// rounding needs no launches of its own.  `fp32`: the caller asked for single-precision iterations, which only
// the large tiles have, so they win earlier.  Measured crossovers of a whole call, T = 300 (ms, small / large
// fp64 / large fp32): M = 32: 3072 blocks 0.259 / 0.280 / 0.216, 3328 blocks 0.314 / 0.286 / 0.222, 2048 blocks
// 0.189 / 0.198 / 0.188; M = 16: 8192 blocks 0.165 / 0.202 / 0.182, 9216 blocks 0.209 / 0.258 / 0.196, 32 768
// blocks 0.484 / 0.492 / 0.367, 65 536 blocks 0.916 / 0.886 / 0.567; M = 8: 12 288 blocks 0.102 / 0.104 / 0.101,
// 16 384 blocks 0.128 / 0.107 / 0.102; M = 4: 49 152 blocks 0.085 / 0.104 / 0.095, 57 344 blocks 0.107 / 0.106 /
// 0.097, 81 920 blocks 0.133 / 0.174 / 0.113, 131 072 blocks 0.199 / 0.186 / 0.126.
constexpr int64_t small_tiles_below_blocks(int M, bool fp32) {
  return M == 4 ? (fp32 ? 55000 : 100000) : M == 8 ? (fp32 ? 12000 : 13000) : M == 16 ? (fp32 ? 9000 : 40000)
       : M == 32 ? (fp32 ? 2100 : 3200) : 0;
}

// Below this many blocks in a launch the greedy selection runs with M lanes per block: the one-lane kernel
// takes the time of M*M dependent steps of a single wave however few blocks there are (22 / 70 / 310 us for
// M = 16 / 32 / 64), the M-lane kernel issues several times the instructions but its chain is M steps, so it
// wins while it does not fill the chip.  Measured crossovers (us, one lane / M lanes, T = 300): M = 32: 8192
// blocks 70 / 52, 12 288 blocks 70 / 69, 16 384 blocks 70 / 84; M = 16: 12 288 blocks 22 / 20, 16 384 blocks
// 23 / 25; M = 64: 8192 blocks 308 / 214, 12 288 blocks 317 / 315, 16 384 blocks 314 / 396.  For M <= 8 the
// one-lane kernel is never slower.
constexpr int64_t greedy_wide_below_blocks(int M) { return M == 16 ? 14000 : M == 32 ? 12000 : M == 64 ? 12000 : 0; }

// Enqueues the kernels of one fused launch that depend on M: tile load + Algorithm 1 + sort, greedy selection
// (or the simple rounding arm), local search + mask write.  `b.count` non-degenerate problems of variant v.
// ev (optional): events recorded after the first and the second of the three.
// Returns false if a launch could not be described (more workgroups than a grid holds).
template <int M>
bool launch_block_kernels(Batch& b, const Variant& v, hipStream_t stream, hipEvent_t ev_sorted, hipEvent_t ev_greedy);

extern template bool launch_block_kernels<4>(Batch&, const Variant&, hipStream_t, hipEvent_t, hipEvent_t);
extern template bool launch_block_kernels<8>(Batch&, const Variant&, hipStream_t, hipEvent_t, hipEvent_t);
extern template bool launch_block_kernels<16>(Batch&, const Variant&, hipStream_t, hipEvent_t, hipEvent_t);
extern template bool launch_block_kernels<32>(Batch&, const Variant&, hipStream_t, hipEvent_t, hipEvent_t);
extern template bool launch_block_kernels<64>(Batch&, const Variant&, hipStream_t, hipEvent_t, hipEvent_t);

}  // namespace tsenor_dev
