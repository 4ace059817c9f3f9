// Selection step and subgraph step of Algorithm 1 for a small partition, in one launch.
//
// The general path spends six launches per epoch on these two steps, each a few microseconds long
// whatever the size; for a partition of a few thousand entries that is a third of the whole
// training step.  Here one workgroup of 1024 threads runs the same stages back to back, with a
// barrier where the general path has a kernel boundary (a barrier also publishes the workgroup's
// earlier global writes to its own threads).  The keep bits and the per-word prefix of the kept
// count stay in LDS, so the rank of a boundary node is two LDS reads and a population count.
// Every output is an integer array with a unique value: both paths write the same bits.
#include "device_utils.hpp"
#include "kernels.hpp"

namespace bns {

namespace {

constexpr int kSmallThreads = 1024;
constexpr int kSmallWords = kSmallMaxHalo / kWave;

struct SmallArgs {
  // selection step
  const int64_t *halo_gid;
  int32_t n_halo;
  uint32_t k0, k1, epoch;
  const uint32_t *epoch_dev;
  uint32_t part_id;
  uint64_t threshold;
  uint64_t *ballots;
  int32_t *kept_ids, *remap, *n_kept, *kept_start;
  // subgraph step
  int32_t n_in, e_in, e_bd;
  StaticSplit sp;
  int32_t *kpos, *row_ptr, *col_idx, *nnz;
  // transposed rows of the kept nodes
  const int32_t *halo_ptr, *halo_col;
  int32_t *t_tail_ptr, *t_col_idx;
};

__global__ void __launch_bounds__(kSmallThreads) sample_build_small_kernel(const SmallArgs a) {
  __shared__ uint64_t words[kSmallWords];      // keep bits, one word per 64 boundary nodes
  __shared__ int word_prefix[kSmallWords + 1];  // kept nodes before each word; [n_words] = all
  __shared__ int kept_b[kSmallMaxHalo];         // the kept list
  __shared__ int kept_pos[kSmallMaxHalo];       // where each kept node's transposed row starts
  const int t = threadIdx.x, lane = lane_id();
  const uint32_t epoch = a.epoch_dev ? *a.epoch_dev : a.epoch;
  const int n_words = (a.n_halo + kWave - 1) / kWave;

  // ---- keep bits -------------------------------------------------------------------------------
  for (int b0 = 0; b0 < a.n_halo; b0 += kSmallThreads) {  // trip count uniform over the block
    const int b = b0 + t;
    bool keep = false;
    if (b < a.n_halo) {
      const uint64_t gid = (uint64_t)a.halo_gid[b];
      uint32_t c0 = (uint32_t)gid, c1 = (uint32_t)(gid >> 32), c2 = epoch, c3 = a.part_id;
      philox4x32_10(c0, c1, c2, c3, a.k0, a.k1);
      keep = (uint64_t)c0 < a.threshold;
    }
    const uint64_t word = __ballot(keep);
    if (lane == 0 && b < a.n_halo) {
      words[b >> 6] = word;
      a.ballots[b >> 6] = word;
    }
  }
  __syncthreads();
  {
    const int c = t < n_words ? __popcll(words[t]) : 0;
    int total;
    const int before = block_exclusive_scan<kSmallThreads>(c, &total);
    if (t < n_words) word_prefix[t] = before;
    if (t == 0) {
      word_prefix[n_words] = total;
      *a.n_kept = total;
    }
  }
  __syncthreads();
  const int n_kept = word_prefix[n_words];
  auto rank_of = [&](int b) -> int {  // rank of a kept boundary node
    return word_prefix[b >> 6] + __popcll(words[b >> 6] & ((1ull << (b & 63)) - 1ull));
  };

  // ---- kept list, remap ------------------------------------------------------------------------
  for (int b = t; b < a.n_halo; b += kSmallThreads) {
    if ((words[b >> 6] >> (b & 63)) & 1ull) {
      const int r = rank_of(b);
      kept_b[r] = b;
      a.kept_ids[r] = b;
      a.remap[b] = r;
    } else {
      a.remap[b] = -1;
    }
  }
  __syncthreads();

  // ---- rows of the kept nodes in the transposed subgraph: starts = prefix sum of list lengths ----
  int run = a.e_in;
  for (int r0 = 0; r0 < n_kept; r0 += kSmallThreads) {
    const int r = r0 + t;
    int len = 0;
    if (r < n_kept) {
      const int b = kept_b[r];
      len = a.halo_ptr[b + 1] - a.halo_ptr[b];
    }
    int sum;
    const int before = block_exclusive_scan<kSmallThreads>(len, &sum);
    if (r < n_kept) {
      kept_pos[r] = run + before;
      a.kept_start[r] = run + before;
      a.t_tail_ptr[r] = run + before;
    }
    run += sum;
  }
  if (t == 0) {
    a.kept_start[n_kept] = run;
    a.t_tail_ptr[n_kept] = run;
  }
  __syncthreads();
  for (int i = t; i < n_kept * 8; i += kSmallThreads) {  // eight lanes copy one list
    const int r = i >> 3, sub = i & 7;
    const int b = kept_b[r];
    const int src = a.halo_ptr[b], len = a.halo_ptr[b + 1] - src;
    const int dst = kept_pos[r];
    for (int k = sub; k < len; k += 8) a.t_col_idx[dst + k] = a.halo_col[src + k];
  }

  // ---- boundary entries: kpos = kept boundary entries before each one; kept ones to their place --
  run = 0;
  for (int k0 = 0; k0 < a.e_bd; k0 += kSmallThreads) {
    const int k = k0 + t;
    int b = 0;
    bool kept = false;
    if (k < a.e_bd) {
      b = a.sp.bd_b[k];
      kept = (words[b >> 6] >> (b & 63)) & 1ull;
    }
    int sum;
    const int pos = run + block_exclusive_scan<kSmallThreads>(kept ? 1 : 0, &sum);
    if (k < a.e_bd) {
      a.kpos[k] = pos;
      if (kept) a.col_idx[a.sp.inner_ptr[a.sp.bd_row[k] + 1] + pos] = a.n_in + rank_of(b);
    }
    run += sum;
  }
  if (t == 0 && a.e_bd > 0) a.kpos[a.e_bd] = run;
  __syncthreads();  // kpos is read below by other threads than its writers

  // ---- row starts and inner entries --------------------------------------------------------------
  for (int v = t; v <= a.n_in; v += kSmallThreads) {
    const int r = a.sp.inner_ptr[v] + (a.e_bd > 0 ? a.kpos[a.sp.bd_ptr[v]] : 0);
    a.row_ptr[v] = r;
    if (v == a.n_in) *a.nnz = r;
  }
  for (int j = t; j < a.e_in; j += kSmallThreads)
    a.col_idx[j + (a.e_bd > 0 ? a.kpos[a.sp.in_bdp[j]] : 0)] = a.sp.in_col[j];
}

}  // namespace

bool sample_build_small_fits(int32_t n_in, int32_t n_halo, int64_t e_in, int64_t e_bd) {
  return n_halo <= kSmallMaxHalo && e_bd <= kSmallMaxBoundaryEntries &&
         (int64_t)n_in + e_in <= kSmallMaxInnerWork;
}

hipError_t sample_build_small(const int64_t *halo_gid, int32_t n_halo, uint64_t seed, uint32_t epoch,
                              const uint32_t *epoch_dev, uint32_t part_id, uint64_t threshold, uint64_t *ballots,
                              int32_t *kept_ids, int32_t *remap, int32_t *n_kept, int32_t *kept_start,
                              int32_t n_in, int64_t e_in, int64_t e_bd, const StaticSplit &sp, int32_t *kpos,
                              int32_t *row_ptr, int32_t *col_idx, int32_t *nnz, const int32_t *halo_ptr,
                              const int32_t *halo_col, int32_t *t_row_ptr, int32_t *t_col_idx, hipStream_t s) {
  if (!sample_build_small_fits(n_in, n_halo, e_in, e_bd)) return hipErrorInvalidValue;
  SmallArgs a;
  a.halo_gid = halo_gid;
  a.n_halo = n_halo;
  a.k0 = (uint32_t)seed;
  a.k1 = (uint32_t)(seed >> 32);
  a.epoch = epoch;
  a.epoch_dev = epoch_dev;
  a.part_id = part_id;
  a.threshold = threshold;
  a.ballots = ballots;
  a.kept_ids = kept_ids;
  a.remap = remap;
  a.n_kept = n_kept;
  a.kept_start = kept_start;
  a.n_in = n_in;
  a.e_in = (int32_t)e_in;
  a.e_bd = (int32_t)e_bd;
  a.sp = sp;
  a.kpos = kpos;
  a.row_ptr = row_ptr;
  a.col_idx = col_idx;
  a.nnz = nnz;
  a.halo_ptr = halo_ptr;
  a.halo_col = halo_col;
  a.t_tail_ptr = t_row_ptr + n_in;
  a.t_col_idx = t_col_idx;
  sample_build_small_kernel<<<1, kSmallThreads, 0, s>>>(a);
  return hipGetLastError();
}

}  // namespace bns
