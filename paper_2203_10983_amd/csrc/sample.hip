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
// number of kept nodes per tile (tile_sums[tile], raw counts).  With halo_ptr (the boundary
// nodes' static lists of inner neighbours) also the summed list length of the tile's kept nodes
// (tile_sums[tiles + tile]): the rows of the kept nodes in the transposed subgraph are laid out in
// kept order, so their starts are a prefix sum of exactly these lengths.
__global__ void __launch_bounds__(kSampleThreads)
sample_flags_kernel(const int64_t *__restrict__ halo_gid, int32_t n_halo, uint32_t k0, uint32_t k1,
                    uint32_t epoch, const uint32_t *__restrict__ epoch_dev, uint32_t part_id,
                    uint64_t threshold, const int32_t *__restrict__ halo_ptr, uint64_t *__restrict__ ballots,
                    int32_t *__restrict__ tile_sums) {
  if (epoch_dev) epoch = *epoch_dev;  // epoch counter kept on the device (graph replay)
  const int lane = lane_id();
  int cnt = 0, len = 0;
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
    if (keep && halo_ptr) len += halo_ptr[b + 1] - halo_ptr[b];
  }
  __shared__ int red[2][kSampleThreads / kWave];
  cnt = wave_sum(cnt);
  len = wave_sum(len);
  if (lane == 0) {
    red[0][threadIdx.x / kWave] = cnt;
    red[1][threadIdx.x / kWave] = len;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int total = 0, len_total = 0;
#pragma unroll
    for (int w = 0; w < kSampleThreads / kWave; ++w) {
      total += red[0][w];
      len_total += red[1][w];
    }
    tile_sums[blockIdx.x] = total;
    if (halo_ptr) tile_sums[gridDim.x + blockIdx.x] = len_total;
  }
}

// Pass 2: rank of every kept node = kept nodes in earlier tiles (summed by the block itself) +
// kept nodes in earlier words of the tile + kept lanes below it in its own word.  The tile's kept
// nodes are first compacted into LDS in rank order; the block then walks the ranks, so that
// kept_ids is written with consecutive addresses and (with halo_ptr) the start of each kept node's
// row in the transposed subgraph, first + the list lengths of the kept nodes before it, comes from a
// block scan over just the kept ones: kept_start[rank], and kept_start[n_kept] = the end.
// Block 0 also writes the totals.
__global__ void __launch_bounds__(kSampleThreads)
sample_write_kernel(int32_t n_halo, const uint64_t *__restrict__ ballots,
                    const int32_t *__restrict__ tile_counts, int32_t *__restrict__ kept_ids,
                    int32_t *__restrict__ remap, int32_t *__restrict__ n_kept,
                    const int32_t *__restrict__ halo_ptr, int32_t first, int32_t *__restrict__ kept_start) {
  __shared__ int word_prefix[kWordsPerTile + 1];
  __shared__ int kept_b[kScanTile];
  const int lane = lane_id();
  int total = 0, len_total = 0;
  const int base = tiles_before<kSampleThreads>(tile_counts, blockIdx.x, gridDim.x, blockIdx.x == 0 ? &total : nullptr);
  int run = first;
  if (halo_ptr)
    run += tiles_before<kSampleThreads>(tile_counts + gridDim.x, blockIdx.x, gridDim.x,
                                        blockIdx.x == 0 ? &len_total : nullptr);
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    *n_kept = total;
    if (halo_ptr) kept_start[total] = first + len_total;
  }
  const int64_t word0 = (int64_t)blockIdx.x * kWordsPerTile;
  const int64_t n_words = ((int64_t)n_halo + kWave - 1) / kWave;
  if (threadIdx.x < kWave) {
    const int64_t w = word0 + threadIdx.x;
    const int c = (threadIdx.x < kWordsPerTile && w < n_words) ? __popcll(ballots[w]) : 0;
    const int inc = wave_inclusive_scan(c);
    if (threadIdx.x < kWordsPerTile) word_prefix[threadIdx.x] = inc - c;
    if (threadIdx.x == kWordsPerTile - 1) word_prefix[kWordsPerTile] = inc;  // kept nodes of the tile
  }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < kSampleIters; ++it) {
    const int local = it * kSampleThreads + threadIdx.x;
    const int64_t b = (int64_t)blockIdx.x * kScanTile + local;
    if (b < n_halo) {
      const uint64_t word = ballots[b >> 6];
      if ((word >> lane) & 1ull) {
        const int r = word_prefix[local >> 6] + __popcll(word & ((1ull << lane) - 1ull));
        kept_b[r] = (int32_t)b;
        remap[b] = base + r;
      } else {
        remap[b] = -1;
      }
    }
  }
  __syncthreads();
  const int tile_kept = word_prefix[kWordsPerTile];
  for (int r0 = 0; r0 < tile_kept; r0 += kSampleThreads) {  // block-uniform trip count
    const int r = r0 + threadIdx.x;
    const int b = r < tile_kept ? kept_b[r] : -1;
    if (b >= 0) kept_ids[base + r] = b;
    if (halo_ptr) {
      const int len = b >= 0 ? halo_ptr[b + 1] - halo_ptr[b] : 0;
      int sum;
      const int before = block_exclusive_scan<kSampleThreads>(len, &sum);
      if (b >= 0) kept_start[base + r] = run + before;
      run += sum;
    }
  }
}

hipError_t sample_boundary(const int64_t *halo_gid, int32_t n_halo, uint64_t seed, uint32_t epoch,
                           const uint32_t *epoch_dev, uint32_t part_id, uint64_t threshold, uint64_t *ballots,
                           int32_t *tile_sums, int32_t *kept_ids, int32_t *remap, int32_t *n_kept,
                           const int32_t *halo_ptr, int32_t first, int32_t *kept_start, hipStream_t s) {
  if (!kept_start) halo_ptr = nullptr;
  const int nb = scan_tiles(n_halo) > 0 ? scan_tiles(n_halo) : 1;
  sample_flags_kernel<<<nb, kSampleThreads, 0, s>>>(halo_gid, n_halo, (uint32_t)seed,
                                                    (uint32_t)(seed >> 32), epoch, epoch_dev, part_id,
                                                    threshold, halo_ptr, ballots, tile_sums);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  sample_write_kernel<<<nb, kSampleThreads, 0, s>>>(n_halo, ballots, tile_sums, kept_ids, remap, n_kept,
                                                    halo_ptr, first, kept_start);
  return hipGetLastError();
}

}  // namespace bns
