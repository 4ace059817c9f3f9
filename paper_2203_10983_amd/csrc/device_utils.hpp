// Device helpers shared by the gfx950 kernels: 64-lane wavefront scans and reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bns {

constexpr int kWave = 64;

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// Inclusive prefix sum over the 64 lanes of a wavefront.
__device__ __forceinline__ int wave_inclusive_scan(int x) {
  const int lane = lane_id();
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    int y = __shfl_up(x, off, kWave);
    if (lane >= off) x += y;
  }
  return x;
}

__device__ __forceinline__ int wave_sum(int x) {
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) x += __shfl_xor(x, off, kWave);
  return x;
}

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) x += __shfl_xor(x, off, kWave);
  return x;
}

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) x = fmaxf(x, __shfl_xor(x, off, kWave));
  return x;
}

// Exclusive prefix sum of one int per thread over a block of NT threads (NT multiple of 64,
// NT <= 1024).  Returns the exclusive prefix; *block_total receives the sum on every thread.
template <int NT>
__device__ __forceinline__ int block_exclusive_scan(int x, int *block_total) {
  __shared__ int wave_tot[NT / kWave];
  const int lane = lane_id(), wid = threadIdx.x / kWave;
  const int inc = wave_inclusive_scan(x);
  if (lane == kWave - 1) wave_tot[wid] = inc;
  __syncthreads();
  int base = 0, total = 0;
#pragma unroll
  for (int w = 0; w < NT / kWave; ++w) {
    const int t = wave_tot[w];
    if (w < wid) base += t;
    total += t;
  }
  __syncthreads();
  *block_total = total;
  return base + inc - x;
}

}  // namespace bns
