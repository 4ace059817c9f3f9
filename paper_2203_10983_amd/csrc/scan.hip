// Device-wide exclusive prefix sum of int32 (three short kernels: tile sums, scan of the tile
// sums by one block, per-tile scan + offset).  The element count may live on the device.
#include "device_utils.hpp"
#include "kernels.hpp"

namespace bns {

constexpr int kScanThreads = 256;
constexpr int kScanItems = kScanTile / kScanThreads;  // 8 contiguous elements per thread

__global__ void __launch_bounds__(kScanThreads)
scan_tile_sums_kernel(const int32_t *__restrict__ in, int64_t n_max, const int32_t *n_dev,
                      int32_t *__restrict__ tile_sums) {
  const int64_t n = n_dev ? (int64_t)*n_dev : n_max;
  const int64_t tile0 = (int64_t)blockIdx.x * kScanTile;
  int sum = 0;
  if (tile0 < n) {
    const int64_t i0 = tile0 + (int64_t)threadIdx.x * kScanItems;
#pragma unroll
    for (int k = 0; k < kScanItems; ++k)
      if (i0 + k < n) sum += in[i0 + k];
  }
  int total;
  block_exclusive_scan<kScanThreads>(sum, &total);
  if (threadIdx.x == 0) tile_sums[blockIdx.x] = total;
}

// One block turns sums[0..nb) into exclusive prefixes in place; sums[nb] and *total_out = total.
__global__ void __launch_bounds__(1024)
scan_sums_kernel(int32_t *__restrict__ sums, int nb, int32_t *total_out) {
  int carry = 0;
  for (int base = 0; base < nb; base += 1024) {
    const int i = base + threadIdx.x;
    const int x = i < nb ? sums[i] : 0;
    int total;
    const int ex = block_exclusive_scan<1024>(x, &total);
    if (i < nb) sums[i] = carry + ex;
    carry += total;
  }
  if (threadIdx.x == 0) {
    sums[nb] = carry;
    if (total_out) *total_out = carry;
  }
}

__global__ void __launch_bounds__(kScanThreads)
scan_tile_apply_kernel(const int32_t *__restrict__ in, int32_t *__restrict__ out, int64_t n_max,
                       const int32_t *n_dev, const int32_t *__restrict__ tile_sums,
                       int32_t add_base) {
  const int64_t n = n_dev ? (int64_t)*n_dev : n_max;
  const int64_t tile0 = (int64_t)blockIdx.x * kScanTile;
  if (n == 0 && blockIdx.x == 0 && threadIdx.x == 0) out[0] = add_base;
  if (tile0 >= n) return;
  const int64_t i0 = tile0 + (int64_t)threadIdx.x * kScanItems;
  int v[kScanItems];
  int sum = 0;
#pragma unroll
  for (int k = 0; k < kScanItems; ++k) {
    v[k] = (i0 + k < n) ? in[i0 + k] : 0;
    sum += v[k];
  }
  int total;
  int run = add_base + tile_sums[blockIdx.x] + block_exclusive_scan<kScanThreads>(sum, &total);
#pragma unroll
  for (int k = 0; k < kScanItems; ++k) {
    if (i0 + k < n) {
      out[i0 + k] = run;
      run += v[k];
      if (i0 + k == n - 1) out[n] = run;
    }
  }
}

hipError_t scan_exclusive_i32(const int32_t *in, int32_t *out, int64_t n_max, const int32_t *n_dev,
                              int32_t *tile_sums, int32_t *total_out, int32_t add_base,
                              hipStream_t s) {
  const int nb = scan_tiles(n_max) > 0 ? scan_tiles(n_max) : 1;
  scan_tile_sums_kernel<<<nb, kScanThreads, 0, s>>>(in, n_max, n_dev, tile_sums);
  scan_sums_kernel<<<1, 1024, 0, s>>>(tile_sums, nb, total_out);
  scan_tile_apply_kernel<<<nb, kScanThreads, 0, s>>>(in, out, n_max, n_dev, tile_sums, add_base);
  return hipGetLastError();
}

}  // namespace bns
