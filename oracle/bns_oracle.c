/*
 * CPU oracle for one partition's BNS-GCN training step  --  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, fp64 implementation of what the step computes, written from
 * the paper (Algorithm 1; Section 3.2 "Boundary Node Sampling"; Appendix A,
 * the propagation matrix P and the sampled form with the diagonal matrix S).
 * It shares no code with the HIP library and must never be called from the
 * product path: only tests, the smoke check and the benchmark's CPU-baseline
 * leg load it.  No blocking, no fusion, no reordering: each function is the
 * definition written out as loops (OpenMP only splits independent rows).
 *
 * Integer outputs are exact; floating point is fp64 throughout.  Inputs that
 * are fp32 by definition (features, boundary features, weights) are widened
 * on read, which is exact.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int bnso_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ------------------------------------------------------------------------- *
 * Counter-based random draw.  The paper only says "randomly pick elements of
 * B_i with probability p" (Algorithm 1, selection step); the generator is this
 * build's choice: Philox-4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw,
 * "Parallel random numbers: as easy as 1, 2, 3", SC'11).
 *   counter = (gid low word, gid high word, epoch, partition id)
 *   key     = (seed low word, seed high word)
 *   draw    = first output word.
 * ------------------------------------------------------------------------- */
void bnso_philox4x32_10(const uint32_t ctr_in[4], const uint32_t key_in[2], uint32_t out[4]) {
  uint32_t c0 = ctr_in[0], c1 = ctr_in[1], c2 = ctr_in[2], c3 = ctr_in[3];
  uint32_t k0 = key_in[0], k1 = key_in[1];
  for (int round = 0; round < 10; ++round) {
    if (round > 0) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }   /* Weyl key schedule */
    uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    uint32_t n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

uint32_t bnso_draw(uint64_t seed, uint32_t epoch, uint32_t part_id, uint64_t gid) {
  uint32_t ctr[4] = {(uint32_t)gid, (uint32_t)(gid >> 32), epoch, part_id};
  uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t out[4];
  bnso_philox4x32_10(ctr, key, out);
  return out[0];
}

/* keep  <=>  draw < floor(p * 2^32), an integer comparison (p = 1 keeps all, p = 0 none). */
uint64_t bnso_threshold(double p) { return (uint64_t)floor(p * 4294967296.0); }

/* Algorithm 1, selection step: U = { b in B : kept }, each b independently.
 * kept_ids lists U ascending; remap[b] = rank of b in U, or -1.  Returns |U|. */
int64_t bnso_sample(uint64_t seed, uint32_t epoch, uint32_t part_id, double p,
                    const int64_t *halo_gid, int64_t n_halo, int32_t *kept_ids, int32_t *remap) {
  const uint64_t T = bnso_threshold(p);
  int64_t n_kept = 0;
  for (int64_t b = 0; b < n_halo; ++b) {
    uint64_t u = bnso_draw(seed, epoch, part_id, (uint64_t)halo_gid[b]);
    if (u < T) { kept_ids[n_kept] = (int32_t)b; remap[b] = (int32_t)n_kept; ++n_kept; }
    else remap[b] = -1;
  }
  return n_kept;
}

/* Dropout on hidden activations (Section 4 trains with dropout; the element-wise draw is this
 * build's reading): element (row, col) of the output of hidden layer `layer` is kept with
 * probability 1 - q.  One draw per element, built like the boundary draw: the first output word
 * of Philox-4x32-10 on the counter (row, col, part_id * 256 + layer, epoch) under the key
 * (seed lo, seed hi xor 0x64726F70), a stream separate from the boundary draw;
 * keep  <=>  word < floor((1 - q) * 2^32). */
void bnso_dropout_mask(uint64_t seed, uint32_t epoch, uint32_t part_id, uint32_t layer,
                       int64_t n_rows, int64_t n_cols, double q, uint8_t *keep) {
  const uint64_t T = bnso_threshold(1.0 - q);
  const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32) ^ 0x64726F70u};
#pragma omp parallel for schedule(static)
  for (int64_t row = 0; row < n_rows; ++row) {
    for (int64_t col = 0; col < n_cols; ++col) {
      uint32_t ctr[4] = {(uint32_t)row, (uint32_t)col, (part_id << 8) | layer, epoch};
      uint32_t out[4];
      bnso_philox4x32_10(ctr, key, out);
      keep[row * n_cols + col] = (uint64_t)out[0] < T ? 1 : 0;
    }
  }
}

/* Algorithm 1, subgraph step: node-induced subgraph on V u U.  Inner columns stay,
 * boundary column n_in+b stays iff b in U and becomes n_in+rank(b); order kept. */
int64_t bnso_induced_csr(int64_t n_in, const int32_t *row_ptr0, const int32_t *col0,
                         const int32_t *remap, int32_t *row_ptr, int32_t *col_idx) {
  int64_t nnz = 0;
  row_ptr[0] = 0;
  for (int64_t v = 0; v < n_in; ++v) {
    for (int64_t e = row_ptr0[v]; e < row_ptr0[v + 1]; ++e) {
      int32_t c = col0[e];
      if (c < n_in) col_idx[nnz++] = c;
      else if (remap[c - n_in] >= 0) col_idx[nnz++] = (int32_t)(n_in + remap[c - n_in]);
    }
    row_ptr[v + 1] = (int32_t)nnz;
  }
  return nnz;
}

/* Transpose of an n_rows x n_cols CSR pattern by a stable counting sort. */
void bnso_transpose(int64_t n_rows, int64_t n_cols, const int32_t *row_ptr, const int32_t *col_idx,
                    int32_t *t_row_ptr, int32_t *t_col_idx) {
  int64_t nnz = row_ptr[n_rows];
  memset(t_row_ptr, 0, (size_t)(n_cols + 1) * sizeof(int32_t));
  for (int64_t e = 0; e < nnz; ++e) t_row_ptr[col_idx[e] + 1]++;
  for (int64_t c = 0; c < n_cols; ++c) t_row_ptr[c + 1] += t_row_ptr[c];
  int32_t *cursor = (int32_t *)malloc((size_t)(n_cols + 1) * sizeof(int32_t));
  memcpy(cursor, t_row_ptr, (size_t)(n_cols + 1) * sizeof(int32_t));
  for (int64_t v = 0; v < n_rows; ++v)
    for (int64_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e) t_col_idx[cursor[col_idx[e]]++] = (int32_t)v;
  free(cursor);
}

/* d~^{-1/2} of stacked column u of the sampled subgraph (full-graph degrees, Appendix A). */
static inline double dis_of(int64_t u, int64_t n_in, const int32_t *deg_in, const int32_t *deg_halo,
                            const int32_t *kept_ids) {
  return u < n_in ? 1.0 / sqrt((double)deg_in[u]) : 1.0 / sqrt((double)deg_halo[kept_ids[u - n_in]]);
}

/* Aggregate (Eq. 1 in the sampled matrix form of Appendix A):
 *   A[v,:] = sum_{u in row v} P_vu * S_uu * Hcat[u,:],   P_vu = d~_v^{-1/2} d~_u^{-1/2},
 *   S_uu = 1 for inner u, s_halo (= 1/p) for kept boundary u,
 *   Hcat = [H_in ; halo_h[kept_ids]]. */
void bnso_aggregate(int64_t n_in, int64_t d, const int32_t *row_ptr, const int32_t *col_idx,
                    const int32_t *deg_in, const int32_t *deg_halo, const int32_t *kept_ids,
                    double s_halo, const double *H_in, const float *halo_h, double *A) {
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t v = 0; v < n_in; ++v) {
    double *a = A + v * d;
    for (int64_t j = 0; j < d; ++j) a[j] = 0.0;
    const double dv = dis_of(v, n_in, deg_in, deg_halo, kept_ids);
    for (int64_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e) {
      const int64_t u = col_idx[e];
      const double du = dis_of(u, n_in, deg_in, deg_halo, kept_ids);
      if (u < n_in) {
        const double w = dv * du;
        const double *h = H_in + u * d;
        for (int64_t j = 0; j < d; ++j) a[j] += w * h[j];
      } else {
        const double w = dv * du * s_halo;
        const float *h = halo_h + (int64_t)kept_ids[u - n_in] * d;
        for (int64_t j = 0; j < d; ++j) a[j] += w * (double)h[j];
      }
    }
  }
}

/* Backward of the aggregate: dHcat = S^T P^T dA, through the transposed pattern
 * (t_row_ptr/t_col_idx: stacked column u -> rows v holding u).
 *   u inner:          dH_in[u,:]        = d~_u^{-1/2} * sum_v d~_v^{-1/2} dA[v,:]
 *   u kept boundary:  dhalo[u - n_in,:] = s_halo * d~_u^{-1/2} * sum_v d~_v^{-1/2} dA[v,:] */
void bnso_aggregate_bwd(int64_t n_in, int64_t n_kept, int64_t d, const int32_t *t_row_ptr,
                        const int32_t *t_col_idx, const int32_t *deg_in, const int32_t *deg_halo,
                        const int32_t *kept_ids, double s_halo, const double *dA, double *dH_in,
                        double *dhalo) {
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t u = 0; u < n_in + n_kept; ++u) {
    double *g = u < n_in ? dH_in + u * d : dhalo + (u - n_in) * d;
    for (int64_t j = 0; j < d; ++j) g[j] = 0.0;
    for (int64_t e = t_row_ptr[u]; e < t_row_ptr[u + 1]; ++e) {
      const int64_t v = t_col_idx[e];
      const double dv = 1.0 / sqrt((double)deg_in[v]);
      const double *a = dA + v * d;
      for (int64_t j = 0; j < d; ++j) g[j] += dv * a[j];
    }
    const double su = dis_of(u, n_in, deg_in, deg_halo, kept_ids) * (u < n_in ? 1.0 : s_halo);
    for (int64_t j = 0; j < d; ++j) g[j] *= su;
  }
}

/* ------------------------------------------------------------------------- *
 * GraphSAGE with a mean aggregator (Section 2: zeta = mean over the neighbours,
 * phi = sigma(W . CONCAT(z_v, h_v))), the instance the paper trains.  Under
 * boundary sampling the received boundary features are divided by p
 * (Section 3.2, "for a mean aggregator we replace H with H/p"), and the mean
 * keeps the FULL-graph neighbour count, so that the estimate is unbiased:
 *   z_v = ( sum_{inner u ~ v} h_u + (1/p) sum_{kept boundary u ~ v} h_u ) / deg_v ,
 * deg_v = number of neighbours of v in the whole graph (no self-loop).  The
 * stored pattern carries one self-loop per row; the mean skips it.
 * ------------------------------------------------------------------------- */
void bnso_aggregate_mean(int64_t n_in, int64_t d, const int32_t *row_ptr, const int32_t *col_idx,
                         const int32_t *deg_in, const int32_t *kept_ids, double s_halo,
                         const double *H_in, const float *halo_h, double *Z) {
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t v = 0; v < n_in; ++v) {
    double *z = Z + v * d;
    for (int64_t j = 0; j < d; ++j) z[j] = 0.0;
    for (int64_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e) {
      const int64_t u = col_idx[e];
      if (u == v) continue; /* the self-loop is not a neighbour */
      if (u < n_in) {
        const double *h = H_in + u * d;
        for (int64_t j = 0; j < d; ++j) z[j] += h[j];
      } else {
        const float *h = halo_h + (int64_t)kept_ids[u - n_in] * d;
        for (int64_t j = 0; j < d; ++j) z[j] += s_halo * (double)h[j];
      }
    }
    const int64_t deg = (int64_t)deg_in[v] - 1; /* deg_in counts the self-loop */
    const double inv = deg > 0 ? 1.0 / (double)deg : 0.0;
    for (int64_t j = 0; j < d; ++j) z[j] *= inv;
  }
}

/* Backward of the mean aggregate through the transposed pattern:
 *   u inner:          dH_in[u,:]        = sum_{v ~ u, v != u} dZ[v,:] / deg_v
 *   u kept boundary:  dhalo[u - n_in,:] = s_halo * sum_{v ~ u} dZ[v,:] / deg_v          */
void bnso_aggregate_mean_bwd(int64_t n_in, int64_t n_kept, int64_t d, const int32_t *t_row_ptr,
                             const int32_t *t_col_idx, const int32_t *deg_in, double s_halo,
                             const double *dZ, double *dH_in, double *dhalo) {
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t u = 0; u < n_in + n_kept; ++u) {
    double *g = u < n_in ? dH_in + u * d : dhalo + (u - n_in) * d;
    for (int64_t j = 0; j < d; ++j) g[j] = 0.0;
    for (int64_t e = t_row_ptr[u]; e < t_row_ptr[u + 1]; ++e) {
      const int64_t v = t_col_idx[e];
      if (v == u) continue;
      const int64_t deg = (int64_t)deg_in[v] - 1;
      const double inv = deg > 0 ? 1.0 / (double)deg : 0.0;
      const double *a = dZ + v * d;
      for (int64_t j = 0; j < d; ++j) g[j] += inv * a[j];
    }
    if (u >= n_in)
      for (int64_t j = 0; j < d; ++j) g[j] *= s_halo;
  }
}
