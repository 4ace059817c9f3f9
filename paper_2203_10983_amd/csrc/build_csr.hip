// Node-induced subgraph on the inner nodes plus the kept boundary nodes (Algorithm 1, subgraph
// step), as a canonical CSR, and its transpose for the backward pass.
//
// Columns are ascending in a row, so the boundary entries are each row's tail.  Once, at set-up,
// the static CSR is split into its inner entries and its boundary entries (both row-major, each
// with its row).  Per epoch only the boundary entries are filtered (the work is proportional to
// the number of boundary edges, Appendix D): an entry-parallel prefix sum over their keep flags
// gives every kept boundary entry, every inner entry and every row start its final position
// without any per-row loop, so power-law rows cost nothing extra.
//
//   kpos[k]     = kept boundary entries before boundary entry k            (prefix sum)
//   row_ptr[v]  = inner_ptr[v] + kpos[bd_ptr[v]]
//   inner entry j of row v      -> col_idx[j + kpos[bd_ptr[v]]]
//   kept boundary entry k, row v -> col_idx[inner_ptr[v+1] + kpos[k]]
#include <algorithm>

#include "device_utils.hpp"
#include "kernels.hpp"

namespace bns {

constexpr int kThreads = 256;

// ---------------------------------------------------------------------------------- set-up
__global__ void __launch_bounds__(kThreads)
count_inner_kernel(int32_t n_in, const int32_t *__restrict__ row_ptr0,
                   const int32_t *__restrict__ col0, int32_t *__restrict__ n_inner) {
  const int v = blockIdx.x * kThreads + threadIdx.x;
  if (v >= n_in) return;
  int lo = row_ptr0[v], hi = row_ptr0[v + 1];
  const int start = lo;
  while (lo < hi) {  // first entry whose column is a boundary column
    const int mid = (lo + hi) >> 1;
    if (col0[mid] < n_in) lo = mid + 1; else hi = mid;
  }
  n_inner[v] = lo - start;
}

// One wavefront per row scatters the row's entries into the inner and boundary lists.
__global__ void __launch_bounds__(kThreads)
split_entries_kernel(int32_t n_in, const int32_t *__restrict__ row_ptr0,
                     const int32_t *__restrict__ col0, const int32_t *__restrict__ inner_ptr,
                     int32_t *__restrict__ bd_ptr, int32_t *__restrict__ in_col,
                     int32_t *__restrict__ in_bdp, int32_t *__restrict__ bd_b,
                     int32_t *__restrict__ bd_row) {
  const int lane = lane_id();
  const int waves = gridDim.x * (kThreads / kWave);
  for (int v = blockIdx.x * (kThreads / kWave) + threadIdx.x / kWave; v <= n_in; v += waves) {
    if (v == n_in) {
      if (lane == 0) bd_ptr[n_in] = row_ptr0[n_in] - inner_ptr[n_in];
      continue;
    }
    const int e0 = row_ptr0[v], e1 = row_ptr0[v + 1];
    const int i0 = inner_ptr[v], ni = inner_ptr[v + 1] - i0;
    const int b0 = e0 - i0;
    if (lane == 0) bd_ptr[v] = b0;
    for (int e = e0 + lane; e < e1; e += kWave) {
      const int c = col0[e];
      const int o = e - e0;
      if (o < ni) { in_col[i0 + o] = c; in_bdp[i0 + o] = b0; }
      else { bd_b[b0 + o - ni] = c - n_in; bd_row[b0 + o - ni] = v; }
    }
  }
}

__global__ void __launch_bounds__(kThreads)
degree_rsqrt_kernel(const int32_t *__restrict__ deg, int32_t n, float *__restrict__ dis) {
  const int i = blockIdx.x * kThreads + threadIdx.x;
  if (i < n) dis[i] = 1.0f / sqrtf((float)deg[i]);
}

__global__ void __launch_bounds__(kThreads)
degree_inverse_kernel(const int32_t *__restrict__ deg, int32_t n, float *__restrict__ inv) {
  const int i = blockIdx.x * kThreads + threadIdx.x;
  if (i < n) inv[i] = deg[i] > 1 ? 1.0f / (float)(deg[i] - 1) : 0.f;
}

hipError_t degree_inverse(const int32_t *deg, int32_t n, float *inv, hipStream_t s) {
  if (n > 0) degree_inverse_kernel<<<(n + kThreads - 1) / kThreads, kThreads, 0, s>>>(deg, n, inv);
  return hipGetLastError();
}

hipError_t degree_rsqrt(const int32_t *deg, int32_t n, float *dis, hipStream_t s) {
  if (n > 0) degree_rsqrt_kernel<<<(n + kThreads - 1) / kThreads, kThreads, 0, s>>>(deg, n, dis);
  return hipGetLastError();
}

hipError_t build_static_split(int32_t n_in, const int32_t *row_ptr0, const int32_t *col0,
                              const StaticSplit &sp, int32_t *tile_sums, hipStream_t s) {
  count_inner_kernel<<<(n_in + kThreads - 1) / kThreads, kThreads, 0, s>>>(n_in, row_ptr0, col0,
                                                                           sp.n_inner);
  hipError_t e = scan_exclusive_i32(sp.n_inner, sp.inner_ptr, n_in, nullptr, tile_sums, nullptr, 0, s);
  if (e != hipSuccess) return e;
  const int blocks = (n_in + 1 + (kThreads / kWave) - 1) / (kThreads / kWave);
  split_entries_kernel<<<blocks < 65536 ? blocks : 65536, kThreads, 0, s>>>(
      n_in, row_ptr0, col0, sp.inner_ptr, sp.bd_ptr, sp.in_col, sp.in_bdp, sp.bd_b, sp.bd_row);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------- per epoch
// The keep decision of a boundary node is one bit of the sampler's ballot words (a table of
// n_halo/8 bytes that stays in L2); the 4-byte rank is only fetched for kept entries.
__device__ __forceinline__ bool kept_bit(const uint64_t *__restrict__ ballots, int b) {
  return (ballots[b >> 6] >> (b & 63)) & 1ull;
}

// A tile of kScanTile boundary entries per workgroup; every wavefront owns a contiguous piece of
// it and walks the piece 64 entries at a time, so that all reads and the kpos writes are
// consecutive over the lanes.  The keep flags of a pass are one ballot word; positions inside a
// pass come from the population count of the lower lanes' bits.
constexpr int kWavesPerBlock = kThreads / kWave;
constexpr int kPasses = kScanTile / kThreads;  // passes of 64 entries per wavefront

__global__ void __launch_bounds__(kThreads)
bd_keep_tile_sums_kernel(int64_t e_bd, const int32_t *__restrict__ bd_b,
                         const uint64_t *__restrict__ ballots, int32_t *__restrict__ tile_sums) {
  __shared__ int wave_cnt[kWavesPerBlock];
  const int lane = lane_id(), wid = threadIdx.x / kWave;
  const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)wid * (kPasses * kWave);
  int cnt = 0;
#pragma unroll
  for (int i = 0; i < kPasses; ++i) {
    const int64_t k = base + i * kWave + lane;
    const bool kept = k < e_bd && kept_bit(ballots, bd_b[k]);
    cnt += __popcll(__ballot(kept));
  }
  if (lane == 0) wave_cnt[wid] = cnt;
  __syncthreads();
  if (threadIdx.x == 0) {
    int total = 0;
#pragma unroll
    for (int w = 0; w < kWavesPerBlock; ++w) total += wave_cnt[w];
    tile_sums[blockIdx.x] = total;
  }
}

__global__ void __launch_bounds__(kThreads)
bd_fill_kernel(int32_t n_in, int64_t e_bd, const int32_t *__restrict__ bd_b,
               const int32_t *__restrict__ bd_row, const uint64_t *__restrict__ ballots,
               const int32_t *__restrict__ remap, const int32_t *__restrict__ tile_counts, const int32_t *__restrict__ inner_ptr,
               int32_t *__restrict__ kpos, int32_t *__restrict__ col_idx) {
  __shared__ int wave_cnt[kWavesPerBlock];
  const int lane = lane_id(), wid = threadIdx.x / kWave;
  // kept boundary entries in the tiles before this one: summed here from the raw per-tile counts
  const int tile_offset = tiles_before<kThreads>(tile_counts, blockIdx.x, gridDim.x, nullptr);
  const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)wid * (kPasses * kWave);
  int b[kPasses];
  unsigned long long mask[kPasses];
  int cnt = 0;
#pragma unroll
  for (int i = 0; i < kPasses; ++i) {
    const int64_t k = base + i * kWave + lane;
    b[i] = k < e_bd ? bd_b[k] : -1;
    mask[i] = __ballot(b[i] >= 0 && kept_bit(ballots, b[i]));
    cnt += __popcll(mask[i]);
  }
  if (lane == 0) wave_cnt[wid] = cnt;
  __syncthreads();
  int run = tile_offset;  // kept boundary entries before this wavefront's piece
  for (int w = 0; w < wid; ++w) run += wave_cnt[w];
  const unsigned long long lower = (1ull << lane) - 1ull;
#pragma unroll
  for (int i = 0; i < kPasses; ++i) {
    const int64_t k = base + i * kWave + lane;
    const bool kept = (mask[i] >> lane) & 1ull;
    const int pos = run + __popcll(mask[i] & lower);
    if (k < e_bd) {
      kpos[k] = pos;
      if (kept) col_idx[inner_ptr[bd_row[k] + 1] + pos] = n_in + remap[b[i]];
      if (k == e_bd - 1) kpos[e_bd] = pos + (kept ? 1 : 0);
    }
    run += __popcll(mask[i]);
  }
}

// Row starts and the inner entries in one launch: both follow in closed form from kpos (row v's
// entries move down by the kept boundary entries of the rows before it, kpos[bd_ptr[v]]; every
// inner entry carries its row's bd_ptr, so it needs one gather).
__global__ void __launch_bounds__(kThreads)
finish_csr_kernel(int32_t n_in, int64_t e_in, int64_t e_bd, const int32_t *__restrict__ inner_ptr,
                  const int32_t *__restrict__ bd_ptr, const int32_t *__restrict__ kpos,
                  const int32_t *__restrict__ in_col, const int32_t *__restrict__ in_bdp,
                  int32_t *__restrict__ row_ptr, int32_t *__restrict__ col_idx, int32_t *__restrict__ nnz) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  const int64_t t0 = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  for (int64_t v = t0; v <= n_in; v += stride) {
    const int r = inner_ptr[v] + (e_bd > 0 ? kpos[bd_ptr[v]] : 0);
    row_ptr[v] = r;
    if (v == n_in) *nnz = r;
  }
  for (int64_t j = t0; j < e_in; j += stride) col_idx[j + (e_bd > 0 ? kpos[in_bdp[j]] : 0)] = in_col[j];
}

hipError_t build_sampled_csr(int32_t n_in, int64_t e_in, int64_t e_bd, const StaticSplit &sp,
                             const uint64_t *ballots, const int32_t *remap, int32_t *kpos, int32_t *tile_sums,
                             int32_t *row_ptr, int32_t *col_idx, int32_t *nnz, hipStream_t s) {
  if (e_bd > 0) {
    const int nb = scan_tiles(e_bd);
    bd_keep_tile_sums_kernel<<<nb, kThreads, 0, s>>>(e_bd, sp.bd_b, ballots, tile_sums);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    bd_fill_kernel<<<nb, kThreads, 0, s>>>(n_in, e_bd, sp.bd_b, sp.bd_row, ballots, remap, tile_sums,
                                           sp.inner_ptr, kpos, col_idx);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  int64_t blocks = (std::max<int64_t>(e_in, (int64_t)n_in + 1) + kThreads * 4 - 1) / (kThreads * 4);
  if (blocks < 1) blocks = 1;
  finish_csr_kernel<<<(unsigned)blocks, kThreads, 0, s>>>(n_in, e_in, e_bd, sp.inner_ptr, sp.bd_ptr, kpos, sp.in_col,
                                                          sp.in_bdp, row_ptr, col_idx, nnz);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------- transpose
// Rows of the kept boundary nodes in the transposed CSR: kept node r (boundary node b =
// kept_ids[r]) gets b's static list of inner neighbours.  Where each row starts was settled by the
// sampler (a prefix sum of the list lengths in kept order, kept_start[0..n_kept]); eight lanes copy
// one list and write the row's start.
__global__ void __launch_bounds__(kThreads)
kept_rows_fill_kernel(const int32_t *__restrict__ n_kept, const int32_t *__restrict__ kept_ids,
                      const int32_t *__restrict__ halo_ptr, const int32_t *__restrict__ halo_col,
                      const int32_t *__restrict__ kept_start, int32_t *__restrict__ t_tail_ptr,
                      int32_t *__restrict__ t_col_idx) {
  const int r = (blockIdx.x * kThreads + threadIdx.x) >> 3;
  const int sub = threadIdx.x & 7;
  const int n = *n_kept;
  if (r == 0 && sub == 0) t_tail_ptr[n] = kept_start[n];
  if (r >= n) return;
  const int b = kept_ids[r];
  const int src = halo_ptr[b], len = halo_ptr[b + 1] - src;
  const int dst = kept_start[r];
  if (sub == 0) t_tail_ptr[r] = dst;
  for (int i = sub; i < len; i += 8) t_col_idx[dst + i] = halo_col[src + i];
}

__global__ void __launch_bounds__(kThreads)
copy_static_kernel(const int32_t *__restrict__ a_src, int64_t a_n, int32_t *__restrict__ a_dst,
                   const int32_t *__restrict__ b_src, int64_t b_n, int32_t *__restrict__ b_dst) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < a_n + b_n; i += stride) {
    if (i < a_n) a_dst[i] = a_src[i];
    else b_dst[i - a_n] = b_src[i - a_n];
  }
}

hipError_t build_transposed_csr(int32_t n_in, int32_t n_halo, int64_t e_in,
                                const int32_t *t_in_ptr, const int32_t *t_in_col,
                                const int32_t *halo_ptr, const int32_t *halo_col,
                                const int32_t *kept_ids, const int32_t *n_kept,
                                const int32_t *kept_start, int32_t *t_row_ptr, int32_t *t_col_idx,
                                bool static_rows, bool kept_rows, hipStream_t s) {
  // rows of inner nodes never change: the transpose of the inner-inner block (copied by a kernel,
  // so that the whole step stays a plain chain of kernel nodes under graph capture)
  if (static_rows) {
    const int64_t n4 = ((int64_t)n_in + 1 + e_in + 3) / 4;
    int64_t blocks = (n4 + kThreads - 1) / kThreads;
    if (blocks > 16384) blocks = 16384;
    copy_static_kernel<<<(unsigned)blocks, kThreads, 0, s>>>(t_in_ptr, (int64_t)n_in + 1, t_row_ptr, t_in_col,
                                                            e_in, t_col_idx);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (n_halo == 0 || !kept_rows) return hipSuccess;
  // rows of kept boundary nodes: their static lists of inner neighbours, in kept order
  const int64_t threads = (int64_t)n_halo * 8;
  kept_rows_fill_kernel<<<(unsigned)((threads + kThreads - 1) / kThreads), kThreads, 0, s>>>(
      n_kept, kept_ids, halo_ptr, halo_col, kept_start, t_row_ptr + n_in, t_col_idx);
  return hipGetLastError();
}

}  // namespace bns
