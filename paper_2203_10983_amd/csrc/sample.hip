// Boundary-node sampling (Algorithm 1, selection step): every boundary node is kept
// independently with probability p, decided by a counter-based draw so that the decision
// depends only on (seed, epoch, partition, global node id).  Kept nodes are compacted in
// ascending order with wavefront ballots and prefix sums.
#include "device_utils.hpp"
#include "kernels.hpp"

namespace bns {

// First output word of the Philox draw.
__device__ __forceinline__ uint32_t philox4x32_10_word0(uint32_t c0, uint32_t c1, uint32_t c2,
                                                        uint32_t c3, uint32_t k0, uint32_t k1) {
  philox4x32_10(c0, c1, c2, c3, k0, k1);
  return c0;
}

constexpr int kSampleThreads = 256;
constexpr int kSampleIters = kScanTile / kSampleThreads;  // 8 wave-words per wave and tile
constexpr int kWordsPerTile = kScanTile / kWave;          // 32

// Pass 1: keep flags as one 64-bit ballot word per 64 consecutive boundary nodes, and the
// number of kept nodes per tile (tile_sums[tile], raw counts).
__global__ void __launch_bounds__(kSampleThreads)
sample_flags_kernel(const int64_t *__restrict__ halo_gid, int32_t n_halo, uint32_t k0, uint32_t k1,
                    uint32_t epoch, const uint32_t *__restrict__ epoch_dev, uint32_t part_id,
                    uint64_t threshold, uint64_t *__restrict__ ballots, int32_t *__restrict__ tile_sums) {
  if (epoch_dev) epoch = *epoch_dev;  // epoch counter kept on the device (graph replay)
  const int lane = lane_id();
  int cnt = 0;
#pragma unroll
  for (int it = 0; it < kSampleIters; ++it) {
    const int64_t b = (int64_t)blockIdx.x * kScanTile + it * kSampleThreads + threadIdx.x;
    bool keep = false;
    if (b < n_halo) {
      const uint64_t gid = (uint64_t)halo_gid[b];
      const uint32_t u = philox4x32_10_word0((uint32_t)gid, (uint32_t)(gid >> 32), epoch, part_id,
                                             k0, k1);
      keep = (uint64_t)u < threshold;
    }
    const uint64_t word = __ballot(keep);
    if (lane == 0 && b < n_halo) ballots[b >> 6] = word;
    cnt += (lane == 0) ? __popcll(word) : 0;
  }
  int total;
  block_exclusive_scan<kSampleThreads>(cnt, &total);
  if (threadIdx.x == 0) tile_sums[blockIdx.x] = total;
}

// Pass 2: rank of every kept node = kept nodes in earlier tiles (summed by the block itself) +
// kept nodes in earlier words of the tile + kept lanes below it in its own word.  Block 0 also
// writes the total.
__global__ void __launch_bounds__(kSampleThreads)
sample_write_kernel(int32_t n_halo, const uint64_t *__restrict__ ballots,
                    const int32_t *__restrict__ tile_counts, int32_t *__restrict__ kept_ids,
                    int32_t *__restrict__ remap, int32_t *__restrict__ n_kept) {
  __shared__ int word_prefix[kWordsPerTile];
  const int lane = lane_id();
  int total = 0;
  const int base = tiles_before<kSampleThreads>(tile_counts, blockIdx.x, gridDim.x, blockIdx.x == 0 ? &total : nullptr);
  if (blockIdx.x == 0 && threadIdx.x == 0) *n_kept = total;
  const int64_t word0 = (int64_t)blockIdx.x * kWordsPerTile;
  const int64_t n_words = ((int64_t)n_halo + kWave - 1) / kWave;
  if (threadIdx.x < kWave) {
    const int64_t w = word0 + threadIdx.x;
    const int c = (threadIdx.x < kWordsPerTile && w < n_words) ? __popcll(ballots[w]) : 0;
    const int inc = wave_inclusive_scan(c);
    if (threadIdx.x < kWordsPerTile) word_prefix[threadIdx.x] = inc - c;
  }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < kSampleIters; ++it) {
    const int local = it * kSampleThreads + threadIdx.x;
    const int64_t b = (int64_t)blockIdx.x * kScanTile + local;
    if (b < n_halo) {
      const uint64_t word = ballots[b >> 6];
      if ((word >> lane) & 1ull) {
        const int rank = base + word_prefix[local >> 6] + __popcll(word & ((1ull << lane) - 1ull));
        kept_ids[rank] = (int32_t)b;
        remap[b] = rank;
      } else {
        remap[b] = -1;
      }
    }
  }
}

hipError_t sample_boundary(const int64_t *halo_gid, int32_t n_halo, uint64_t seed, uint32_t epoch,
                           const uint32_t *epoch_dev, uint32_t part_id, uint64_t threshold, uint64_t *ballots,
                           int32_t *tile_sums, int32_t *kept_ids, int32_t *remap, int32_t *n_kept,
                           hipStream_t s) {
  const int nb = scan_tiles(n_halo) > 0 ? scan_tiles(n_halo) : 1;
  sample_flags_kernel<<<nb, kSampleThreads, 0, s>>>(halo_gid, n_halo, (uint32_t)seed,
                                                    (uint32_t)(seed >> 32), epoch, epoch_dev, part_id,
                                                    threshold, ballots, tile_sums);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  sample_write_kernel<<<nb, kSampleThreads, 0, s>>>(n_halo, ballots, tile_sums, kept_ids, remap, n_kept);
  return hipGetLastError();
}

}  // namespace bns
