// Measurement aid (not part of the library): issue rate of single vector instructions on the GPU at hand.
//
// The Dykstra kernels are bound by vector-ALU issue, so what an instruction costs decides their form.  Each
// test runs one instruction kind in 12 independent dependency chains per lane, 2 waves per SIMD on every SIMD
// of the chip, and reports the time per wave-instruction per SIMD and the lane-operations per second.
// Bare instructions (inline asm) so that the compiler cannot change what is measured.  Registers only: the
// one store at the end keeps the chains alive.
//
// Build: hipcc --offload-arch=gfx950 -O3 -o issue_rate_probe issue_rate_probe.hip   Run: ./issue_rate_probe
#include <hip/hip_runtime.h>

#include <cstdio>

#define CK(x)                                                                 \
  do {                                                                        \
    hipError_t e_ = (x);                                                      \
    if (e_ != hipSuccess) {                                                   \
      std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
      return 1;                                                               \
    }                                                                         \
  } while (0)

enum Kind {
  FMA32, MUL32, ADD32, MIN32, MAX32, MED3_32, MULCLAMP32, XOR32, MOVDPP, CNDMASK, RCP32,
  FMA64, MUL64, ADD64, MIN64, MAX64, MULCLAMP64, CMP64, RCP64
};

constexpr int kChains = 12, kUnroll = 8, kIters = 3000, kWavesPerSimd = 2;

template <int KIND>
__global__ __launch_bounds__(256) void chain_kernel(float* out, int iters) {
  float x[kChains];
  double d[kChains];
#pragma unroll
  for (int k = 0; k < kChains; ++k) {
    x[k] = (float)(threadIdx.x + k) * 1e-3f;
    d[k] = x[k];
  }
  float a = 1.0000001f, b = 1e-9f;
  double da = 1.0000001, db = 1e-9;
  unsigned long long mask = 0x5555555555555555ull + (unsigned long long)iters;
  asm volatile("" : "+v"(a), "+v"(b), "+v"(da), "+v"(db), "+s"(mask));
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int r = 0; r < kUnroll; ++r)
#pragma unroll
      for (int k = 0; k < kChains; ++k) {
        if constexpr (KIND == FMA32) asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(x[k]) : "v"(a), "v"(b));
        if constexpr (KIND == MUL32) asm volatile("v_mul_f32_e32 %0, %0, %1" : "+v"(x[k]) : "v"(a));
        if constexpr (KIND == ADD32) asm volatile("v_add_f32_e32 %0, %0, %1" : "+v"(x[k]) : "v"(b));
        if constexpr (KIND == MIN32) asm volatile("v_min_f32_e32 %0, %0, %1" : "+v"(x[k]) : "v"(a));
        if constexpr (KIND == MAX32) asm volatile("v_max_f32_e32 %0, %0, %1" : "+v"(x[k]) : "v"(a));
        if constexpr (KIND == MED3_32) asm volatile("v_med3_f32 %0, %0, %1, %2" : "+v"(x[k]) : "v"(a), "v"(b));
        if constexpr (KIND == MULCLAMP32) asm volatile("v_mul_f32_e64 %0, %0, %1 clamp" : "+v"(x[k]) : "v"(a));
        if constexpr (KIND == XOR32) asm volatile("v_xor_b32_e32 %0, %0, %1" : "+v"(x[k]) : "v"(a));
        if constexpr (KIND == MOVDPP)
          asm volatile("v_mov_b32_dpp %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf" : "+v"(x[k]));
        if constexpr (KIND == CNDMASK) asm volatile("v_cndmask_b32_e64 %0, %0, %1, %2" : "+v"(x[k]) : "v"(a), "s"(mask));
        if constexpr (KIND == RCP32) asm volatile("v_rcp_f32_e32 %0, %0" : "+v"(x[k]));
        if constexpr (KIND == FMA64) asm volatile("v_fma_f64 %0, %0, %1, %2" : "+v"(d[k]) : "v"(da), "v"(db));
        if constexpr (KIND == MUL64) asm volatile("v_mul_f64 %0, %0, %1" : "+v"(d[k]) : "v"(da));
        if constexpr (KIND == ADD64) asm volatile("v_add_f64 %0, %0, %1" : "+v"(d[k]) : "v"(db));
        if constexpr (KIND == MIN64) asm volatile("v_min_f64 %0, %0, %1" : "+v"(d[k]) : "v"(da));
        if constexpr (KIND == MAX64) asm volatile("v_max_f64 %0, %0, %1" : "+v"(d[k]) : "v"(da));
        if constexpr (KIND == MULCLAMP64) asm volatile("v_mul_f64 %0, %0, %1 clamp" : "+v"(d[k]) : "v"(da));
        if constexpr (KIND == CMP64) asm volatile("v_cmp_lt_f64_e64 %0, %1, %2" : "=s"(mask) : "v"(d[k]), "v"(da));
        if constexpr (KIND == RCP64) asm volatile("v_rcp_f64_e32 %0, %0" : "+v"(d[k]));
      }
  }
  float s = (float)(mask & 1);
#pragma unroll
  for (int k = 0; k < kChains; ++k) s += x[k] + (float)d[k];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

template <int KIND>
int run(const char* name, int cus) {
  const int blocks = cus * kWavesPerSimd;  // 256 threads: one wave on each of the 4 SIMDs of a CU
  float* out;
  CK(hipMalloc(&out, sizeof(float) * blocks * 256));
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  chain_kernel<KIND><<<blocks, 256>>>(out, 10);
  CK(hipDeviceSynchronize());
  CK(hipEventRecord(e0));
  chain_kernel<KIND><<<blocks, 256>>>(out, kIters);
  CK(hipEventRecord(e1));
  CK(hipEventSynchronize(e1));
  float ms;
  CK(hipEventElapsedTime(&ms, e0, e1));
  const double per_simd = (double)kWavesPerSimd * kIters * kUnroll * kChains;
  std::printf("%-22s %7.3f ms  %5.2f ns per wave-instruction per SIMD  %6.2f T lane-ops/s\n", name, ms, ms * 1e6 / per_simd,
              (double)blocks * 256 * kIters * kUnroll * kChains / (ms * 1e-3) / 1e12);
  std::fflush(stdout);
  CK(hipEventDestroy(e0));
  CK(hipEventDestroy(e1));
  CK(hipFree(out));
  return 0;
}

int main() {
  hipDeviceProp_t prop;
  CK(hipGetDeviceProperties(&prop, 0));
  const int cus = prop.multiProcessorCount;
  std::printf("%s, %d CUs, %d waves per SIMD, %d chains per lane\n", prop.name, cus, kWavesPerSimd, kChains);
  if (run<MUL32>("v_mul_f32", cus)) return 1;
  if (run<ADD32>("v_add_f32", cus)) return 1;
  if (run<FMA32>("v_fma_f32", cus)) return 1;
  if (run<MULCLAMP32>("v_mul_f32 clamp", cus)) return 1;
  if (run<XOR32>("v_xor_b32", cus)) return 1;
  if (run<MIN32>("v_min_f32", cus)) return 1;
  if (run<MAX32>("v_max_f32", cus)) return 1;
  if (run<MED3_32>("v_med3_f32", cus)) return 1;
  if (run<MOVDPP>("v_mov_b32_dpp", cus)) return 1;
  if (run<CNDMASK>("v_cndmask_b32 (sgpr)", cus)) return 1;
  if (run<RCP32>("v_rcp_f32", cus)) return 1;
  if (run<MUL64>("v_mul_f64", cus)) return 1;
  if (run<ADD64>("v_add_f64", cus)) return 1;
  if (run<FMA64>("v_fma_f64", cus)) return 1;
  if (run<MULCLAMP64>("v_mul_f64 clamp", cus)) return 1;
  if (run<MIN64>("v_min_f64", cus)) return 1;
  if (run<MAX64>("v_max_f64", cus)) return 1;
  if (run<CMP64>("v_cmp_lt_f64", cus)) return 1;
  if (run<RCP64>("v_rcp_f64", cus)) return 1;
  return 0;
}
