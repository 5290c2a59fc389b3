// Prefix sums: inclusive over one wave, exclusive over a workgroup of 1024 lanes (16 waves of 64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pipelive {

constexpr int kScanThreads = 1024;

// inclusive prefix sum of `v` over the 64 lanes of a wave
__device__ __forceinline__ int wave_inclusive_scan(int v, int lane) {
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    int t = __shfl_up(v, o);
    if (lane >= o) v += t;
  }
  return v;
}

// returns the exclusive prefix of `v` over threadIdx.x; *total = sum over the workgroup.
// `sh` must hold 17 uint32_t of LDS.  Contains barriers: call from all lanes.
__device__ __forceinline__ uint32_t wg_exclusive_scan(uint32_t v, uint32_t *sh, uint32_t *total) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  uint32_t inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    uint32_t t = __shfl_up(inc, o);
    if (lane >= o) inc += t;
  }
  __syncthreads();  // protect `sh` against the previous use
  if (lane == 63) sh[w] = inc;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t run = 0;
    for (int i = 0; i < kScanThreads / 64; ++i) {
      uint32_t t = sh[i];
      sh[i] = run;
      run += t;
    }
    sh[16] = run;
  }
  __syncthreads();
  *total = sh[16];
  return sh[w] + inc - v;
}

}  // namespace pipelive
