// Device helpers shared by the gfx950 kernels: 64-lane wavefront scans and reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bns {

constexpr int kWave = 64;

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// Philox-4x32 with 10 rounds (Salmon et al., SC'11): multipliers and Weyl key increments as
// published.  The counter words c0..c3 are replaced by the four output words.
__device__ __forceinline__ void philox4x32_10(uint32_t &c0, uint32_t &c1, uint32_t &c2, uint32_t &c3,
                                              uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    const uint32_t n0 = hi1 ^ c1 ^ k0;
    const uint32_t n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
}

// Dropout draw of element (row, col): kept iff the first Philox word on the counter (row, col, c2,
// epoch) is below the threshold.  D: the Dropout parameter block of kernels.hpp.
template <typename D>
__device__ __forceinline__ bool dropout_keeps(const D &drop, int row, int col) {
  uint32_t c0 = (uint32_t)row, c1 = (uint32_t)col, c2 = drop.c2;
  uint32_t c3 = drop.epoch_dev ? *drop.epoch_dev : drop.epoch;
  philox4x32_10(c0, c1, c2, c3, drop.k0, drop.k1);
  return (uint64_t)c0 < drop.threshold;
}

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

// Number of items in the tiles before tile `tile`, from the per-tile counts sums[0..nb): every
// block adds up the counts of its predecessors itself (a few thousand L2-resident integers), which
// saves the separate one-block scan kernel between a counting pass and its consumer.  Every thread
// gets the result; *total (nullable, block-uniform) receives the sum over all nb tiles.
template <int NT>
__device__ __forceinline__ int tiles_before(const int32_t *__restrict__ sums, int tile, int nb, int *total) {
  __shared__ int red[2][NT / kWave];
  int before = 0, all = 0;
  const int n = total ? nb : tile;
  for (int i = threadIdx.x; i < n; i += NT) {
    const int x = sums[i];
    all += x;
    if (i < tile) before += x;
  }
  before = wave_sum(before);
  all = wave_sum(all);
  if (lane_id() == 0) {
    red[0][threadIdx.x / kWave] = before;
    red[1][threadIdx.x / kWave] = all;
  }
  __syncthreads();
  int b = 0, a = 0;
#pragma unroll
  for (int w = 0; w < NT / kWave; ++w) {
    b += red[0][w];
    a += red[1][w];
  }
  __syncthreads();
  if (total) *total = a;
  return b;
}

}  // namespace bns
