// Body of launch_block_kernels<M>: picks the instantiation of every kernel that depends on M and enqueues it.
// Included by exactly one translation unit per M.
#pragma once
#include "dykstra_sort.hpp"
#include "launch.hpp"

namespace tsenor_dev {

// prefix of workgroup counts when every matrix gets ceil(blocks / per_group) workgroups; false on overflow
inline bool assign_groups(Batch& b, int64_t per_group) {
  int64_t total = 0;
  for (int k = 0; k < b.count; ++k) {
    b.first[k] = (unsigned)total;
    total += (b.e[k].p.nblocks + per_group - 1) / per_group;
    if (total > 0x7FFFFFFF) return false;
  }
  for (int k = b.count; k <= kMaxBatch; ++k) b.first[k] = (unsigned)total;
  return true;
}

template <int M>
bool launch_block_kernels(Batch& b, const Variant& v, hipStream_t stream, hipEvent_t ev_sorted, hipEvent_t ev_greedy) {
  constexpr int BPW = kWave >> (Tiling<M>::NX + Tiling<M>::NY);
  int64_t total_blocks = 0;
  for (int k = 0; k < b.count; ++k) total_blocks += b.e[k].p.nblocks;
  constexpr bool kHasSmall = M <= 32;
  const bool small = kHasSmall && !v.fast && !v.zero_t && v.small;
  if (small) {
    // the small tiles carry Algorithm 2 behind the iterations: this one kernel is the whole path
    if constexpr (kHasSmall) {
      constexpr int BPWS = kWave >> (Tiling<M, true>::NX + Tiling<M, true>::NY);
      using L = DykstraLaunch<M, false, false, true>;
      static_assert(L::kWavesPerGroup == 1 && DykstraLaunch<M, false, true, true>::kWavesPerGroup == 1, "");
      if (!assign_groups(b, (int64_t)BPWS)) return false;
      if (v.adaptive)
        dykstra_sort_kernel<M, false, false, true, true><<<b.first[b.count], L::kThreads, 0, stream>>>(b);
      else
        dykstra_sort_kernel<M, false, false, true><<<b.first[b.count], L::kThreads, 0, stream>>>(b);
    }
    if (ev_sorted) (void)hipEventRecord(ev_sorted, stream);
    if (ev_greedy) (void)hipEventRecord(ev_greedy, stream);
    return true;
  } else if (v.fast && v.adaptive) {
    using L = DykstraLaunch<M, true, true>;
    if (!assign_groups(b, (int64_t)BPW * L::kWavesPerGroup)) return false;
    dykstra_sort_kernel<M, true, false, false, true><<<b.first[b.count], L::kThreads, 0, stream>>>(b);
  } else if (v.fast) {
    using L = DykstraLaunch<M, true>;
    if (!assign_groups(b, (int64_t)BPW * L::kWavesPerGroup)) return false;
    dykstra_sort_kernel<M, true><<<b.first[b.count], L::kThreads, 0, stream>>>(b);
  } else {
    using L = DykstraLaunch<M, false>;
    using LA = DykstraLaunch<M, false, true>;
    if (!assign_groups(b, (int64_t)BPW * (v.adaptive ? LA::kWavesPerGroup : L::kWavesPerGroup))) return false;
    if (v.zero_t)
      dykstra_sort_kernel<M, false, true><<<b.first[b.count], L::kThreads, 0, stream>>>(b);
    else if (v.adaptive)
      dykstra_sort_kernel<M, false, false, false, true><<<b.first[b.count], LA::kThreads, 0, stream>>>(b);
    else
      dykstra_sort_kernel<M, false><<<b.first[b.count], L::kThreads, 0, stream>>>(b);
  }
  if (ev_sorted) (void)hipEventRecord(ev_sorted, stream);
  const bool wide = v.greedy ? v.greedy == TSENOR_FLAG_GREEDY_M_LANES : total_blocks < greedy_wide_below_blocks(M);
  if (v.simple) {
    if (!assign_groups(b, kWave)) return false;
    simple_round_kernel<M><<<b.first[b.count], kWave, 0, stream>>>(b);
  } else if (wide) {
    if (!assign_groups(b, kWave / M)) return false;
    greedy_wide_kernel<M><<<b.first[b.count], kWave, 0, stream>>>(b);
  } else {
    if (!assign_groups(b, kWave)) return false;
    constexpr int GW = kGreedyWaves<M>;
    greedy_kernel<M><<<(b.first[b.count] + GW - 1) / GW, kWave * GW, 0, stream>>>(b);
  }
  if (ev_greedy) (void)hipEventRecord(ev_greedy, stream);
  if (!assign_groups(b, kWave / M)) return false;
  finalize_kernel<M><<<b.first[b.count], kWave, 0, stream>>>(b);
  return true;
}

}  // namespace tsenor_dev
