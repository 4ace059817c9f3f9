// Host-side launchers of the gfx950 kernels.  Every launcher enqueues on `s` and returns the
// launch status; none synchronises.  Pointers are device pointers unless named *_host.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bns {

constexpr int kScanTile = 2048;  // elements per block in the scan / compaction kernels
inline int scan_tiles(int64_t n) { return (int)((n + kScanTile - 1) / kScanTile); }

// ---- scan.hip -------------------------------------------------------------------------------
// out[i] = add_base + sum_{j<i} in[j] for i in 0..n (n+1 entries written).  n = *n_dev if n_dev
// is non-null (n <= n_max), else n_max.  tile_sums: scratch int32[scan_tiles(n_max)+1].
// total_out (nullable): receives sum of all n inputs.
hipError_t scan_exclusive_i32(const int32_t *in, int32_t *out, int64_t n_max, const int32_t *n_dev,
                              int32_t *tile_sums, int32_t *total_out, int32_t add_base,
                              hipStream_t s);

// ---- sample.hip (Algorithm 1, selection step) -------------------------------------------------
// ballots: scratch uint64[ceil(B/64)]; tile_sums: scratch int32[2 * scan_tiles(B) + 1] (half of it
// without kept_start).  epoch_dev (nullable): the epoch index is read from device memory instead of
// `epoch`.  halo_ptr + kept_start (both nullable): kept_start[r] = first + the summed lengths
// halo_ptr[b+1] - halo_ptr[b] of the kept nodes before the r-th one, r = 0..n_kept (int32[B+1]): the
// row starts of the kept nodes in the transposed subgraph, which build_transposed_csr reads.
hipError_t sample_boundary(const int64_t *halo_gid, int32_t n_halo, uint64_t seed, uint32_t epoch,
                           const uint32_t *epoch_dev, uint32_t part_id, uint64_t threshold, uint64_t *ballots,
                           int32_t *tile_sums, int32_t *kept_ids, int32_t *remap, int32_t *n_kept,
                           const int32_t *halo_ptr, int32_t first, int32_t *kept_start, hipStream_t s);

// ---- build_csr.hip (Algorithm 1, subgraph step) -----------------------------------------------
struct StaticSplit {       // inner / boundary split of the static CSR, built once
  int32_t *n_inner;        // int32[n_in]       inner entries in row v (scratch of set-up)
  int32_t *inner_ptr;      // int32[n_in+1]     inner entries before row v
  int32_t *bd_ptr;         // int32[n_in+1]     boundary entries before row v
  int32_t *in_col;         // int32[e_in]       inner entries, row-major
  int32_t *in_bdp;         // int32[e_in]       bd_ptr of their rows (boundary entries before the row)
  int32_t *bd_b;           // int32[e_bd]       boundary entries (boundary id), row-major
  int32_t *bd_row;         // int32[e_bd]       their rows
};
hipError_t build_static_split(int32_t n_in, const int32_t *row_ptr0, const int32_t *col0,
                              const StaticSplit &sp, int32_t *tile_sums, hipStream_t s);
hipError_t degree_rsqrt(const int32_t *deg, int32_t n, float *dis, hipStream_t s);

// ballots: the keep bits written by sample_boundary (bit b%64 of word b/64); kpos: scratch
// int32[e_bd+1]; tile_sums: scratch int32[scan_tiles(e_bd)+1].
hipError_t build_sampled_csr(int32_t n_in, int64_t e_in, int64_t e_bd, const StaticSplit &sp,
                             const uint64_t *ballots, const int32_t *remap, int32_t *kpos, int32_t *tile_sums,
                             int32_t *row_ptr, int32_t *col_idx, int32_t *nnz, hipStream_t s);
// kept_start: the row starts of the kept nodes as sample_boundary left them (int32[n_kept+1]).
// static_rows: write the rows of the inner nodes (the transposed inner-inner block, the same every
// epoch: a destination that already holds them can skip it); kept_rows: write the rows of the kept
// boundary nodes.
hipError_t build_transposed_csr(int32_t n_in, int32_t n_halo, int64_t e_in,
                                const int32_t *t_in_ptr, const int32_t *t_in_col,
                                const int32_t *halo_ptr, const int32_t *halo_col,
                                const int32_t *kept_ids, const int32_t *n_kept,
                                const int32_t *kept_start, int32_t *t_row_ptr, int32_t *t_col_idx,
                                bool static_rows, bool kept_rows, hipStream_t s);

// ---- small.hip: selection step + subgraph step of a small partition in one launch -------------
// One workgroup runs the stages of sample_boundary, build_sampled_csr and the kept rows of
// build_transposed_csr back to back and writes the same arrays (t_row_ptr / t_col_idx must already
// hold the static rows of the inner nodes).  Only for sizes within the limits below, where the six
// launches of the general path cost more than the work itself.
constexpr int kSmallMaxHalo = 4096;              // boundary nodes
constexpr int kSmallMaxBoundaryEntries = 8192;   // entries with a boundary column
constexpr int kSmallMaxInnerWork = 16384;        // inner nodes + inner entries
bool sample_build_small_fits(int32_t n_in, int32_t n_halo, int64_t e_in, int64_t e_bd);
hipError_t sample_build_small(const int64_t *halo_gid, int32_t n_halo, uint64_t seed, uint32_t epoch,
                              const uint32_t *epoch_dev, uint32_t part_id, uint64_t threshold, uint64_t *ballots,
                              int32_t *kept_ids, int32_t *remap, int32_t *n_kept, int32_t *kept_start,
                              int32_t n_in, int64_t e_in, int64_t e_bd, const StaticSplit &sp, int32_t *kpos,
                              int32_t *row_ptr, int32_t *col_idx, int32_t *nnz, const int32_t *halo_ptr,
                              const int32_t *halo_col, int32_t *t_row_ptr, int32_t *t_col_idx, hipStream_t s);

struct Dropout;  // defined with the GEMMs below

// ---- spmm.hip (Eq. 1 in the sampled form of Appendix A, and its transpose) ---------------------
constexpr int kSegLen = 256;  // a wavefront aggregates at most this many neighbours
// Static cut of the rows of a CSR pattern into segments of <= kSegLen entries (by the static row
// lengths; a sampled row is never longer).  Upper bounds for sizing, given rows and entries:
//   segments <= rows + nnz/kSegLen, partial slots <= 2*nnz/kSegLen, multi-segment rows <= nnz/kSegLen
struct SegPlan {
  int32_t *seg_ptr;   // int32[n_rows+1] first segment of each row
  int32_t *seg_row;   // int32[n_seg]    row of each segment
  int32_t *part_ptr;  // int32[n_rows+1] first partial-sum slot of each multi-segment row
  int32_t *mrow;      // int32[n_multi]  rows with more than one segment
  int32_t *part_row;  // int32[n_part]   row of each partial-sum slot
  int32_t n_seg, n_part, n_multi;  // host copies of the totals
  int32_t avg_len;                 // entries per row of the static pattern (launch heuristics)
};
inline int64_t seg_max_segments(int64_t rows, int64_t nnz) { return rows + nnz / kSegLen + 1; }
inline int64_t seg_max_parts(int64_t nnz) { return 2 * (nnz / kSegLen) + 2; }
inline int64_t seg_max_multi(int64_t nnz) { return nnz / kSegLen + 1; }
// Fills *plan (its arrays must be allocated to the bounds above) and waits for the stream.
// tmp_a: scratch int32[n_rows], tmp_b: scratch int32[n_rows+1].  nnz: entries of the pattern.
hipError_t build_seg_plan(int32_t n_rows, int64_t nnz, const int32_t *row_ptr, SegPlan *plan, int32_t *tmp_a,
                          int32_t *tmp_b, int32_t *tile_sums, hipStream_t s);

// Hu[r,:] = (s_halo * dis_halo[b]) * halo_h[b,:], b = kept_ids[r], r < *n_kept (dis_halo nullable = 1).
hipError_t halo_gather(const float *halo_h, const int32_t *kept_ids, const int32_t *n_kept,
                       int32_t n_halo, const float *dis_halo, float s_halo, int32_t d, float *Hu,
                       hipStream_t s);
// A[v,:] = row_scale[v] * ( init[v,:] + sum_{u<n_in in row v} w_col[u] H_in[u,:] + sum_{kept r in row v} Hu[r,:] )
// w_col / row_scale nullable (= 1).  GCN layer: both = d~^-1/2; mean aggregator: w_col = null,
// row_scale = 1/degree, skip_self.  plan: segmentation of the static local CSR; partials: scratch
// f32[plan.n_part * d].  part (all optional) restricts every row to entries [skip, skip+take) of
// its list, adds the initial row vector, or skips the stored self-loop.
struct SpmmRowPart {
  const int32_t *row_skip = nullptr;
  const int32_t *row_take = nullptr;
  const float *init = nullptr;
  bool skip_self = false;
  // halo_rec (from halo_records): Hu is then the whole boundary-feature table [n_halo, d] as the
  // caller holds it; kept node r reads its row halo_rec[r].x with weight as_float(halo_rec[r].y)
  const int2 *halo_rec = nullptr;
};
// rec[r] = (kept_ids[r], s_halo * dis_halo[kept_ids[r]]) for r < *n_kept (dis_halo nullable = 1): what the
// aggregate needs to read the kept boundary rows where they are instead of a gathered, scaled copy.
hipError_t halo_records(const int32_t *kept_ids, const int32_t *n_kept, int32_t n_halo, const float *dis_halo,
                        float s_halo, int2 *rec, hipStream_t s);
hipError_t spmm_fwd(const SegPlan &plan, int32_t n_in, int32_t d, const int32_t *row_ptr,
                    const int32_t *col_idx, const float *w_col, const float *row_scale,
                    const float *H_in, const float *Hu, float *partials, float *A,
                    const SpmmRowPart &part, bool long_rows_only, bool relu, hipStream_t s,
                    int32_t d_store = 0);
// d_store (spmm_fwd and spmm_bwd; 0 = d): the sources and partial sums have rows of d floats of which
// only the first d_store count (rows padded to a multiple of 4 floats so that a narrow odd width is
// gathered with 16-byte loads); the outputs are dense [., d_store].  Then d < 128, no mask, no init.
// pad_rows makes such a padded copy (pad columns zero).
hipError_t pad_rows(int32_t n_rows, int32_t d, int32_t ld, const float *src, float *dst, hipStream_t s);
// Aggregate and update of one GCN layer in one kernel (Eq. 1 then Eq. 2): a workgroup aggregates 64
// rows into LDS (and stores them to A, which the backward pass needs), then multiplies the tile by
// W on the matrix cores while other workgroups of the same compute unit keep gathering.  Rows cut
// into several segments must have been finished before by spmm_fwd(..., long_rows_only = true).
// Needs d_in % 4 == 0 and 64 < d_in <= 128 (spmm_gemm_fwd_supported).
// concat_self: the update of the mean-aggregator layer, H_out = act([A | H_in] W) with W [2 d_in, d_out]
// (neighbour half first): the tile is multiplied by W_n, overwritten with the rows' own features and
// multiplied by W_s into the same accumulators; needs d_out <= 256 (spmm_gemm_fwd_concat_supported).
bool spmm_gemm_fwd_supported(int32_t d_in);
bool spmm_gemm_fwd_concat_supported(int32_t d_in, int32_t d_out);
hipError_t spmm_gemm_fwd(const SegPlan &plan, int32_t n_in, int32_t d_in, int32_t d_out, const int32_t *row_ptr,
                         const int32_t *col_idx, const float *w_col, const float *row_scale,
                         const float *H_in, const float *Hu, float *partials, float *A,
                         const SpmmRowPart &part, const float *W, float *H_out, bool relu,
                         const Dropout &drop, hipStream_t s, bool concat_self = false);
// For stacked column u < n_in + *n_kept:  g = sum_{v in t_row u} w_col[v] dA[v,:];
//   u <  n_in: dH_in[u,:] = row_scale[u] * (init[u,:] + g)  (zeroed where mask_src[u,:] <= 0 if given)
//   u >= n_in: dhalo[u-n_in,:] = s_halo * dis_halo[kept_ids[u-n_in]] * g   (skipped if dhalo null)
// row_scale, dis_halo, init nullable.  plan: segmentation of the transposed inner-inner block.
hipError_t spmm_bwd(const SegPlan &plan, int32_t n_in, int32_t n_halo, int32_t d,
                    const int32_t *t_row_ptr, const int32_t *t_col_idx, const int32_t *kept_ids,
                    const int32_t *n_kept, const float *w_col, const float *row_scale,
                    const float *dis_halo, float s_halo, const float *dA, const float *mask_src,
                    const float *init, bool skip_self, float *partials, float *dH_in, float *dhalo,
                    hipStream_t s, int32_t d_store = 0);

// ---- gemm.hip (Eq. 2 and its backward; fp32 MFMA) ----------------------------------------------
// Dropout on a hidden layer's output (training set-up of Section 4): element (row, col) is kept iff
// the first word of Philox-4x32-10 on the counter (row, col, c2, epoch) under key (k0, k1) is below
// `threshold`; kept elements are multiplied by `scale` = 1/(1-q).  scale == 0: no dropout.
struct Dropout {
  uint64_t threshold = 0;
  float scale = 0.f;
  uint32_t k0 = 0, k1 = 0, c2 = 0, epoch = 0;
  const uint32_t *epoch_dev = nullptr;  // nullable: the epoch index is read from device memory
};
// C[M,N] = A[M,K] B[K,N] (+ the previous C if accumulate), then optional ReLU (followed by dropout
// when drop.scale != 0).
// m_dev (nullable): device-side row count, *m_dev <= M; rows past it are not touched.
// ldc: row stride of C (0 = N); without relu / accumulate the columns N..ldc-1 are set to zero.
hipError_t gemm_nn(int32_t M, int32_t N, int32_t K, const float *A, const float *B, float *C,
                   bool relu, bool accumulate, const Dropout &drop, const int32_t *m_dev, hipStream_t s,
                   int32_t ldc = 0);
// C[M,N] = [A1 | A2] B with A1, A2 [M,K_half] and B [2 K_half, N] (the concat update of the mean
// aggregator layer, Section 2), then optional ReLU / dropout.  Needs K_half % 16 == 0.
hipError_t gemm_nn_concat(int32_t M, int32_t N, int32_t K_half, const float *A1, const float *A2,
                          const float *B, float *C, bool relu, const Dropout &drop, hipStream_t s);
// [C1 | C2] = alpha * A[M,K] B[2 N_half,K]^T, C1 and C2 dense [M,N_half].  Needs N_half % 64 == 0.
bool gemm_nt_pair_supported(int32_t N_half);
hipError_t gemm_nt_pair(int32_t M, int32_t N_half, int32_t K, const float *A, const float *B, float *C1,
                        float *C2, float alpha, hipStream_t s);
// inv[i] = deg[i] > 1 ? 1 / (deg[i] - 1) : 0   (deg counts the self-loop)
hipError_t degree_inverse(const int32_t *deg, int32_t n, float *inv, hipStream_t s);
// C[M,N] = alpha * A[M,K] B[N,K]^T.  mask_src (nullable, [M,N]): C is zeroed where mask_src <= 0.
// m_dev (nullable): device-side row count, *m_dev <= M; rows past it are not touched.
hipError_t gemm_nt(int32_t M, int32_t N, int32_t K, const float *A, const float *B, float *C,
                   const float *mask_src, float alpha, const int32_t *m_dev, hipStream_t s);
// C[M,N] = A[K,M]^T B[K,N] with K split over the grid; partials: scratch f32[splits*M*N],
// summed in a fixed order.  splitk_splits() gives the split count used for (M,N,K).
int32_t splitk_splits(int32_t M, int32_t N, int32_t K);
// accumulate: the product is added to C.  k_dev (nullable): device-side depth, *k_dev <= K (the
// partial buffer is still sized by splitk_splits(M, N, K)).
hipError_t gemm_tn_splitk(int32_t M, int32_t N, int32_t K, const float *A, const float *B,
                          float *C, float *partials, bool accumulate, const int32_t *k_dev, hipStream_t s);
// C[2 M, N] = [A | A2]^T B with A, A2 [K, M] (weight gradient of the concat update); needs M % 128 == 0
// and partials sized by splitk_splits(2 M, N, K).
bool gemm_tn_concat_supported(int32_t M_half);
hipError_t gemm_tn_splitk_concat(int32_t M, int32_t N, int32_t K, const float *A, const float *A2, const float *B,
                                 float *C, float *partials, bool accumulate, const int32_t *k_dev,
                                 hipStream_t s);

// ---- loss.hip (Algorithm 1, loss step) ---------------------------------------------------------
constexpr int kLossBlocks = 8192;  // partials: scratch f32[kLossBlocks]
hipError_t loss_softmax_ce(int32_t n, int32_t C, const float *logits, const int32_t *labels,
                           float *dZ, float *partials, float *loss, hipStream_t s);
hipError_t loss_sigmoid_bce(int32_t n, int32_t C, const float *logits, const uint8_t *labels,
                            float *dZ, float *partials, float *loss, hipStream_t s);
// Dropout applied in place to H[n_rows, d] (for layers whose ReLU sits in the aggregate's store).
hipError_t dropout_inplace(int32_t n_rows, int32_t d, float *H, const Dropout &drop, hipStream_t s);
// out = scale * dH where H > 0 else 0
hipError_t relu_mask(int64_t n, const float *dH, const float *H, float scale, float *out, hipStream_t s);
// Adam step t (1-based) on n weights; m, v are the caller's moment buffers.
hipError_t adam_update(int64_t n, float *W, const float *dW, float *m, float *v, float lr, float b1,
                       float b2, float eps, int32_t t, hipStream_t s);
// *counter = value / *counter += 1 (one thread; the device-side epoch index of graph replay)
hipError_t set_counter(uint32_t *counter, uint32_t value, hipStream_t s);
hipError_t bump_counter(uint32_t *counter, hipStream_t s);
// W -= lr * dW  (Algorithm 1, update step)
hipError_t sgd_update(int64_t n, float *W, const float *dW, float lr, hipStream_t s);

}  // namespace bns
