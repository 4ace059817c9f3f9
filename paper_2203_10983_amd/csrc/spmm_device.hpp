// Device code shared by the aggregate kernels (Eq. 1 in the sampled matrix form of Appendix A):
// argument block, the gather of one row segment, and the scale / mask / store of a finished row.
#pragma once
#include "device_utils.hpp"
#include "kernels.hpp"

namespace bns {

typedef float v2f __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));
template <int VEC> struct Vec;
template <> struct Vec<1> { using T = float; };
template <> struct Vec<2> { using T = v2f; };
template <> struct Vec<4> { using T = v4f; };

template <int VEC>
__device__ __forceinline__ void vec_fma(float (&acc)[VEC], float w, const typename Vec<VEC>::T &v) {
  const float *p = reinterpret_cast<const float *>(&v);
#pragma unroll
  for (int i = 0; i < VEC; ++i) acc[i] = fmaf(w, p[i], acc[i]);
}

struct SpmmArgs {
  SegPlan plan;                // static segmentation of rows 0..n_split-1
  const int32_t *n_extra_dev;  // nullable: *n_extra_dev further single-segment rows follow (kept boundary)
  int32_t d;                   // floats per gathered row = row stride of src0, src1 and the partial sums
  const int32_t *row_ptr, *col_idx;
  int32_t n_split;             // columns < n_split read src0 (weight w_col[c]); others src1 (weight 1)
  const float *src0, *src1, *w_col;
  // nullable: src1 is the boundary-feature table as the caller holds it (one row per boundary
  // node) and stacked column n_split + r reads its row halo_rec[r].x with weight
  // as_float(halo_rec[r].y); else src1 holds the kept rows in kept order, already scaled
  const int2 *halo_rec;
  float *partials;             // one d-vector per segment of multi-segment rows
  // output rows < n_split: out0 (scale out_scale0[row], optional mask); others: out1
  float *out0, *out1;
  const float *out_scale0;
  const float *mask_src;
  const int32_t *kept_ids;     // out1 row r is scaled by s_halo * dis_halo[kept_ids[r]]
  const float *dis_halo;
  float s_halo;
  // optional restriction of rows < n_split to a part of their entries, and an initial value:
  const int32_t *row_skip;     // skip the first row_skip[row] entries (nullable)
  const int32_t *row_take;     // then use row_take[row] entries instead of the rest (nullable)
  const float *init;           // out0 row = scale * (init row + sum) (nullable)
  bool skip_self;              // entries with column == row contribute nothing (mean aggregator)
  // feature slicing over the XCDs (n_slices = 1: off).  Workgroups are handed to the 8 XCDs in
  // turn, so workgroup b runs on XCD b % 8; with n_slices = S that XCD only ever touches the
  // d_slice = d / S floats of slice (b % 8) % S of every feature row, and its private L2 holds S
  // times as many distinct rows.
  int32_t n_slices, d_slice;
  bool multi_only;             // work units = segments of the multi-segment rows only
  bool relu;                   // rows < n_split: max(., 0) after the scale (update-first layers)
  // columns stored per output row = row stride of out0 / out1; less than d when the sources are
  // padded to a multiple of 4 floats (then no mask, no init, no slices; read by the NARROW kernels only)
  int32_t d_store;
};

// Argument block of the forward aggregate (the transposed pass fills its own).
inline SpmmArgs spmm_fwd_args(const SegPlan &plan, int32_t n_in, int32_t d, const int32_t *row_ptr,
                              const int32_t *col_idx, const float *w_col, const float *row_scale,
                              const float *H_in, const float *Hu, float *partials, float *A,
                              const SpmmRowPart &part) {
  SpmmArgs a{};
  a.plan = plan; a.n_extra_dev = nullptr; a.d = d; a.d_store = d;
  a.row_ptr = row_ptr; a.col_idx = col_idx; a.n_split = n_in;
  a.src0 = H_in; a.src1 = Hu; a.w_col = w_col; a.partials = partials; a.halo_rec = part.halo_rec;
  a.out0 = A; a.out1 = nullptr; a.out_scale0 = row_scale; a.mask_src = nullptr;
  a.kept_ids = nullptr; a.dis_halo = nullptr; a.s_halo = 0.f;
  a.row_skip = part.row_skip; a.row_take = part.row_take; a.init = part.init;
  a.skip_self = part.skip_self;
  a.n_slices = 1; a.d_slice = d; a.multi_only = false; a.relu = false;
  return a;
}

// Scale, optional ReLU mask and store of one finished row slice held as acc[c][i].
// lds_row (nullable): the finished values are also written there, element iv*VEC+i at lds_row[iv*VEC+i].
// NARROW: the sources are padded (d_store < d), the output rows are dense with d_store columns.
template <int VEC, int MAXCH, bool NARROW = false>
__device__ __forceinline__ void finish_row(const SpmmArgs &a, int row, int sl, int nvec, int d_off,
                                           float (&acc)[MAXCH][VEC], float *lds_row = nullptr) {
  using V = typename Vec<VEC>::T;
  const int d = a.d, ds = NARROW ? (int)a.d_store : d;
  float scale;
  float *out;
  const float *mask = nullptr;
  const float *init = nullptr;
  if (row < a.n_split) {
    if (a.init) init = a.init + (size_t)row * d + d_off;
    scale = a.out_scale0 ? a.out_scale0[row] : 1.f;
    out = a.out0 + (size_t)row * ds + d_off;
    if (a.mask_src) mask = a.mask_src + (size_t)row * d + d_off;
  } else {
    if (a.out1 == nullptr) return;
    const int r = row - a.n_split;
    scale = a.dis_halo ? a.s_halo * a.dis_halo[a.kept_ids[r]] : a.s_halo;
    out = a.out1 + (size_t)r * ds + d_off;
  }
#pragma unroll
  for (int c = 0; c < MAXCH; ++c) {
    const int iv = c * kWave + sl;
    if (iv < nvec) {
      V o;
      float *po = reinterpret_cast<float *>(&o);
#pragma unroll
      for (int i = 0; i < VEC; ++i) po[i] = acc[c][i];
      if (init) {
        const V x0 = reinterpret_cast<const V *>(init)[iv];
        const float *p0 = reinterpret_cast<const float *>(&x0);
#pragma unroll
        for (int i = 0; i < VEC; ++i) po[i] += p0[i];
      }
#pragma unroll
      for (int i = 0; i < VEC; ++i) po[i] *= scale;
      if (a.relu) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) po[i] = fmaxf(po[i], 0.f);
      }
      if (mask) {
        const V m = __builtin_nontemporal_load(reinterpret_cast<const V *>(mask) + iv);  // read once
        const float *pm = reinterpret_cast<const float *>(&m);
#pragma unroll
        for (int i = 0; i < VEC; ++i) po[i] = pm[i] > 0.f ? po[i] : 0.f;
      }
      if constexpr (!NARROW) {
        // streamed out: a non-temporal store leaves the L2 to the feature rows being gathered
        // (measured: 1.7 % of a training step on the largest workload)
        __builtin_nontemporal_store(o, reinterpret_cast<V *>(out) + iv);
      } else {  // padded sources: the output rows are dense and hold the first ds columns
#pragma unroll
        for (int i = 0; i < VEC; ++i)
          if (iv * VEC + i < ds) out[iv * VEC + i] = po[i];
      }
      if (lds_row) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) lds_row[iv * VEC + i] = po[i];
      }
    }
  }
}

// Feature-row address and weight of entry `col` (stacked column index c) of row `row`.
__device__ __forceinline__ void entry_source(const SpmmArgs &a, int row, int c, int d_off,
                                             unsigned long long &p, float &w) {
  const int d = a.d;
  if (c < a.n_split) {
    p = (unsigned long long)(a.src0 + (size_t)c * d + d_off);
    w = a.w_col ? a.w_col[c] : 1.f;
    if (a.skip_self && c == row) w = 0.f;  // the stored self-loop is not a neighbour
  } else if (a.halo_rec) {
    const int2 r = a.halo_rec[c - a.n_split];
    p = (unsigned long long)(a.src1 + (size_t)r.x * d + d_off);
    w = __int_as_float(r.y);
  } else {
    p = (unsigned long long)(a.src1 + (size_t)(c - a.n_split) * d + d_off);
    w = 1.f;
  }
}

// acc += sum over the cnt <= 64 entries held one per lane (address p_l, weight w_l) of
// w * feature row.  The lanes span the feature dimension (VEC floats per lane, MAXCH pieces of 64
// lanes); with LPR < 64 lanes per row the wavefront walks 64/LPR neighbours at once, four steps in
// flight, and every lane group keeps its own partial sums (fold_groups adds them).
template <int VEC, int MAXCH, int LPR>
__device__ __forceinline__ void gather_batch(unsigned long long p_l, float w_l, int cnt, int nvec,
                                             float (&acc)[MAXCH][VEC]) {
  using V = typename Vec<VEC>::T;
  constexpr int EP = kWave / LPR;  // neighbours walked at once
  constexpr int UNR = (MAXCH == 1 && LPR >= 32) ? 8 : 4;
  const int lane = lane_id();
  const int g = lane / LPR, sl = lane % LPR;
  const unsigned p_lo = (unsigned)p_l, p_hi = (unsigned)(p_l >> 32);
  for (int j = 0; j < cnt; j += UNR * EP) {
    V v[UNR][MAXCH];
    float w[UNR];
#pragma unroll
    for (int t = 0; t < UNR; ++t) {
      const int jj = j + t * EP + g;
      const bool valid = jj < cnt;
      unsigned lo, hi;
      float wt;
      if constexpr (EP == 1) {  // jj is uniform over the wavefront
        const int js = __builtin_amdgcn_readfirstlane(jj) & (kWave - 1);
        lo = __builtin_amdgcn_readlane(p_lo, js);
        hi = __builtin_amdgcn_readlane(p_hi, js);
        wt = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, w_l), js));
      } else {
        lo = __shfl(p_lo, jj & (kWave - 1), kWave);
        hi = __shfl(p_hi, jj & (kWave - 1), kWave);
        wt = __shfl(w_l, jj & (kWave - 1), kWave);
      }
      w[t] = valid ? wt : 0.f;
      const V *src = reinterpret_cast<const V *>(((unsigned long long)hi << 32) | lo);
#pragma unroll
      for (int c = 0; c < MAXCH; ++c) {
        const int iv = c * kWave + sl;
        if (valid && iv < nvec) v[t][c] = src[iv];
        else v[t][c] = V{};
      }
    }
#pragma unroll
    for (int t = 0; t < UNR; ++t)
#pragma unroll
      for (int c = 0; c < MAXCH; ++c) vec_fma<VEC>(acc[c], w[t], v[t][c]);
  }
}

// Adds the partial sums of the 64/LPR lane groups; afterwards lane group 0 holds the total.
template <int VEC, int MAXCH, int LPR>
__device__ __forceinline__ void fold_groups(float (&acc)[MAXCH][VEC]) {
  if constexpr (kWave / LPR > 1) {
#pragma unroll
    for (int off = LPR; off < kWave; off <<= 1)
#pragma unroll
      for (int i = 0; i < VEC; ++i) acc[0][i] += __shfl_xor(acc[0][i], off, kWave);
  }
}

// Sum of w * (feature row) over the entries [e0, e1) of `row`, at most a few hundred of them;
// lane group 0 (lanes < LPR) ends up with the result.  d_off / nvec: first feature column and
// number of VEC-pieces handled.
template <int VEC, int MAXCH, int LPR>
__device__ __forceinline__ void gather_segment(const SpmmArgs &a, int row, int e0, int e1, int d_off, int nvec,
                                               float (&acc)[MAXCH][VEC]) {
  const int lane = lane_id();
#pragma unroll
  for (int c = 0; c < MAXCH; ++c)
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[c][i] = 0.f;
  for (int base = e0; base < e1; base += kWave) {
    const int cnt = min(kWave, e1 - base);
    // one neighbour per lane: its feature-row address and weight
    unsigned long long p_l = 0;
    float w_l = 0.f;
    if (lane < cnt) entry_source(a, row, a.col_idx[base + lane], d_off, p_l, w_l);
    gather_batch<VEC, MAXCH, LPR>(p_l, w_l, cnt, nvec, acc);
  }
  fold_groups<VEC, MAXCH, LPR>(acc);
}

}  // namespace bns
