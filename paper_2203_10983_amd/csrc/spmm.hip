// Sparse aggregate (Eq. 1 in the sampled matrix form of Appendix A) and its transpose.
//
// Work unit: one 64-lane wavefront owns one SEGMENT of an output row, at most kSegLen
// neighbours.  Power-law graphs put a large share of all edges into a few very long rows; cutting
// every row into bounded segments keeps the wavefronts balanced.  A row with one segment is
// finished by its wavefront; a row with several gets one partial sum per segment, and a second
// small kernel adds them in ascending order.  No atomics anywhere: the backward pass walks the
// transposed pattern, and every output element is produced in a fixed order.
//
// Inside a segment the lanes span the feature dimension with VEC-wide loads, so every neighbour
// row is read as one contiguous, coalesced piece.  When a feature row needs fewer than 64 lanes
// (LPR = lanes per row < 64) the wavefront walks 64/LPR neighbours at once and folds the partial
// sums at the end.  Column indices and their weights are fetched 64 at a time, one per lane,
// and handed to the loop by cross-lane reads, four neighbours in flight per step.
#include <algorithm>

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
  int32_t d;
  const int32_t *row_ptr, *col_idx;
  int32_t n_split;             // columns < n_split read src0 (weight w_col[c]); others src1 (weight 1)
  const float *src0, *src1, *w_col;
  float *partials;             // one d-vector per segment of multi-segment rows
  // output rows < n_split: out0 (scale out_scale0[row], optional mask); others: out1
  float *out0, *out1;
  const float *out_scale0;
  const float *mask_src;
  float mask_scale;            // factor on the elements that pass the mask
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
};

// Scale, optional ReLU mask and store of one finished row slice held as acc[c][i].
template <int VEC, int MAXCH>
__device__ __forceinline__ void finish_row(const SpmmArgs &a, int row, int sl, int nvec, int d_off,
                                           float (&acc)[MAXCH][VEC]) {
  using V = typename Vec<VEC>::T;
  const int d = a.d;
  float scale;
  float *out;
  const float *mask = nullptr;
  const float *init = nullptr;
  if (row < a.n_split) {
    if (a.init) init = a.init + (size_t)row * d + d_off;
    scale = a.out_scale0 ? a.out_scale0[row] : 1.f;
    out = a.out0 + (size_t)row * d + d_off;
    if (a.mask_src) mask = a.mask_src + (size_t)row * d + d_off;
  } else {
    if (a.out1 == nullptr) return;
    const int r = row - a.n_split;
    scale = a.dis_halo ? a.s_halo * a.dis_halo[a.kept_ids[r]] : a.s_halo;
    out = a.out1 + (size_t)r * d + d_off;
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
      if (mask) {
        const V m = reinterpret_cast<const V *>(mask)[iv];
        const float *pm = reinterpret_cast<const float *>(&m);
#pragma unroll
        for (int i = 0; i < VEC; ++i) po[i] = pm[i] > 0.f ? po[i] * a.mask_scale : 0.f;
      }
      reinterpret_cast<V *>(out)[iv] = o;
    }
  }
}

template <int VEC, int MAXCH, int LPR>
__global__ void __launch_bounds__(256) spmm_kernel(const SpmmArgs a) {
  using V = typename Vec<VEC>::T;
  constexpr int EP = kWave / LPR;  // neighbours walked at once
  constexpr int UNR = 4;
  const int lane = lane_id();
  const int g = lane / LPR, sl = lane % LPR;
  const int d = a.d;
  int nvec = d / VEC, d_off = 0;
  int bid = blockIdx.x, nblk = gridDim.x;
  if (a.n_slices > 1) {  // gridDim.x is a multiple of 8
    const int x = bid & 7, per = 8 / a.n_slices;
    d_off = (x % a.n_slices) * a.d_slice;
    nvec = a.d_slice / VEC;
    bid = (bid >> 3) * per + x / a.n_slices;
    nblk = (nblk >> 3) * per;
  }
  // work units: the static segments, then one unit per kept boundary row (count on the device)
  const int n_units = a.plan.n_seg + (a.n_extra_dev ? *a.n_extra_dev : 0);
  for (int unit = bid * 4 + (threadIdx.x >> 6); unit < n_units; unit += nblk * 4) {
  int row, seg = 0, nseg = 1;
  if (unit < a.plan.n_seg) {
    row = a.plan.seg_row[unit];
    const int s0 = a.plan.seg_ptr[row];
    seg = unit - s0;
    nseg = a.plan.seg_ptr[row + 1] - s0;
  } else {
    row = a.n_split + (unit - a.plan.n_seg);
  }
  int e0 = a.row_ptr[row], e1 = a.row_ptr[row + 1];
  if (row < a.n_split) {
    if (a.row_skip) e0 += a.row_skip[row];
    if (a.row_take) e1 = e0 + a.row_take[row];
  }
  if (nseg > 1) {  // this wavefront's slice of the row as it is in this epoch
    const int chunk = (e1 - e0 + nseg - 1) / nseg;
    e0 = min(e1, e0 + seg * chunk);
    e1 = min(e1, e0 + chunk);
  }

  float acc[MAXCH][VEC];
#pragma unroll
  for (int c = 0; c < MAXCH; ++c)
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[c][i] = 0.f;

  for (int base = e0; base < e1; base += kWave) {
    const int cnt = min(kWave, e1 - base);
    // one neighbour per lane: its feature-row address and weight
    unsigned long long p_l = 0;
    float w_l = 0.f;
    if (lane < cnt) {
      const int c = a.col_idx[base + lane];
      if (c < a.n_split) {
        p_l = (unsigned long long)(a.src0 + (size_t)c * d + d_off);
        w_l = a.w_col ? a.w_col[c] : 1.f;
        if (a.skip_self && c == row) w_l = 0.f;  // the stored self-loop is not a neighbour
      } else {
        p_l = (unsigned long long)(a.src1 + (size_t)(c - a.n_split) * d + d_off);
        w_l = 1.f;
      }
    }
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

  if constexpr (EP > 1) {
#pragma unroll
    for (int off = LPR; off < kWave; off <<= 1)
#pragma unroll
      for (int i = 0; i < VEC; ++i) acc[0][i] += __shfl_xor(acc[0][i], off, kWave);
  }

  if (g != 0) {
    // only the first lane group holds the folded sums
  } else if (nseg == 1) {
    finish_row<VEC, MAXCH>(a, row, sl, nvec, d_off, acc);
  } else {
    V *part = reinterpret_cast<V *>(a.partials + (size_t)(a.plan.part_ptr[row] + seg) * d + d_off);
#pragma unroll
    for (int c = 0; c < MAXCH; ++c) {
      const int iv = c * kWave + sl;
      if (iv < nvec) {
        V o;
        float *po = reinterpret_cast<float *>(&o);
#pragma unroll
        for (int i = 0; i < VEC; ++i) po[i] = acc[c][i];
        part[iv] = o;
      }
    }
  }
  }  // unit loop
}

// Rows cut into several segments: add the partial sums in ascending segment order.
template <int VEC, int MAXCH>
__global__ void __launch_bounds__(256) spmm_combine_kernel(const SpmmArgs a) {
  using V = typename Vec<VEC>::T;
  const int lane = lane_id();
  const int j = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (j >= a.plan.n_multi) return;
  const int row = a.plan.mrow[j];
  const int nseg = a.plan.seg_ptr[row + 1] - a.plan.seg_ptr[row];
  const int d = a.d, nvec = d / VEC;
  const float *part = a.partials + (size_t)a.plan.part_ptr[row] * d;
  float acc[MAXCH][VEC];
#pragma unroll
  for (int c = 0; c < MAXCH; ++c)
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[c][i] = 0.f;
  constexpr int CU = 8;  // partial vectors fetched together; they are still added in ascending order
  for (int s0 = 0; s0 < nseg; s0 += CU) {
    V x[CU][MAXCH];
#pragma unroll
    for (int t = 0; t < CU; ++t) {
      const V *ps = reinterpret_cast<const V *>(part + (size_t)(s0 + t) * d);
#pragma unroll
      for (int c = 0; c < MAXCH; ++c) {
        const int iv = c * kWave + lane;
        x[t][c] = (s0 + t < nseg && iv < nvec) ? ps[iv] : V{};
      }
    }
#pragma unroll
    for (int t = 0; t < CU; ++t)
#pragma unroll
      for (int c = 0; c < MAXCH; ++c) {
        const float *px = reinterpret_cast<const float *>(&x[t][c]);
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[c][i] += px[i];
      }
  }
  finish_row<VEC, MAXCH>(a, row, lane, nvec, 0, acc);
}

template <int VEC>
static hipError_t launch_spmm_vec(const SpmmArgs &a_in, int64_t max_units, hipStream_t s) {
  SpmmArgs a = a_in;
  a.n_slices = 1;
  a.d_slice = a.d;
  // Wide rows are cut into slices of 128 floats (64 where rows are long enough to keep a
  // wavefront busy with a quarter of its lanes per neighbour); measured on the five workloads,
  // narrower slices lose more to the repeated index walk than the L2 gains.
  if (VEC == 4) {
    const int target = a.plan.avg_len >= 64 ? 64 : 128;
    int S = 1;
    while (S < 8 && a.d / (2 * S) >= target && a.d % (2 * S * VEC) == 0) S *= 2;
    a.n_slices = S;
    a.d_slice = a.d / S;
  }
  const int nvec = a.d_slice / VEC;
  const int full_nvec = a.d / VEC;
  // one wavefront per static segment; the kept boundary rows, whose count lives on the device,
  // are strided over by a bounded number of extra blocks (blocks past the count would only cost
  // dispatch time)
  const int64_t seg_blocks = ((int64_t)a.plan.n_seg + 3) / 4;
  const int64_t extra_blocks = std::min<int64_t>((max_units - a.plan.n_seg + 3) / 4, 8192);
  unsigned blocks = (unsigned)(seg_blocks + std::max<int64_t>(extra_blocks, 0));
  const unsigned cblocks = (unsigned)((a.plan.n_multi + 3) / 4);
  if (blocks == 0) return hipSuccess;
  if (a.n_slices > 1) {
    const unsigned per = 8 / a.n_slices;
    blocks = (blocks + per - 1) / per * 8;
  }
#define BNS_SPMM(MAXCH, LPR) spmm_kernel<VEC, MAXCH, LPR><<<blocks, 256, 0, s>>>(a)
  if (nvec <= 1) BNS_SPMM(1, 1);
  else if (nvec <= 2) BNS_SPMM(1, 2);
  else if (nvec <= 4) BNS_SPMM(1, 4);
  else if (nvec <= 8) BNS_SPMM(1, 8);
  else if (nvec <= 16) BNS_SPMM(1, 16);
  else if (nvec <= 32) BNS_SPMM(1, 32);
  else if (nvec <= 64) BNS_SPMM(1, 64);
  else if (nvec <= 128) BNS_SPMM(2, 64);
  else if (nvec <= 256) BNS_SPMM(4, 64);
  else if (nvec <= 384) BNS_SPMM(6, 64);
  else if (nvec <= 512) BNS_SPMM(8, 64);
  else return hipErrorInvalidValue;
#undef BNS_SPMM
  if (cblocks) {
#define BNS_COMBINE(MAXCH) spmm_combine_kernel<VEC, MAXCH><<<cblocks, 256, 0, s>>>(a)
    if (full_nvec <= 64) BNS_COMBINE(1);
    else if (full_nvec <= 128) BNS_COMBINE(2);
    else if (full_nvec <= 256) BNS_COMBINE(4);
    else if (full_nvec <= 384) BNS_COMBINE(6);
    else BNS_COMBINE(8);
#undef BNS_COMBINE
  }
  return hipGetLastError();
}

static hipError_t launch_spmm(const SpmmArgs &a, int64_t max_units, hipStream_t s) {
  if (a.d % 4 == 0) return launch_spmm_vec<4>(a, max_units, s);
  if (a.d % 2 == 0) return launch_spmm_vec<2>(a, max_units, s);
  return launch_spmm_vec<1>(a, max_units, s);
}

hipError_t spmm_fwd(const SegPlan &plan, int32_t n_in, int32_t d, const int32_t *row_ptr,
                    const int32_t *col_idx, const float *w_col, const float *row_scale,
                    const float *H_in, const float *Hu, float *partials, float *A,
                    const SpmmRowPart &part, hipStream_t s) {
  SpmmArgs a{};
  a.plan = plan; a.n_extra_dev = nullptr; a.d = d;
  a.row_ptr = row_ptr; a.col_idx = col_idx; a.n_split = n_in;
  a.src0 = H_in; a.src1 = Hu; a.w_col = w_col; a.partials = partials;
  a.out0 = A; a.out1 = nullptr; a.out_scale0 = row_scale; a.mask_src = nullptr; a.mask_scale = 1.f;
  a.kept_ids = nullptr; a.dis_halo = nullptr; a.s_halo = 0.f;
  a.row_skip = part.row_skip; a.row_take = part.row_take; a.init = part.init;
  a.skip_self = part.skip_self;
  return launch_spmm(a, plan.n_seg, s);
}

hipError_t spmm_bwd(const SegPlan &plan, int32_t n_in, int32_t n_halo, int32_t d,
                    const int32_t *t_row_ptr, const int32_t *t_col_idx, const int32_t *kept_ids,
                    const int32_t *n_kept, const float *w_col, const float *row_scale,
                    const float *dis_halo, float s_halo, const float *dA, const float *mask_src,
                    float mask_scale, const float *init, bool skip_self, float *partials, float *dH_in,
                    float *dhalo, hipStream_t s) {
  SpmmArgs a{};
  const bool halo_rows = dhalo && n_halo > 0;
  a.plan = plan; a.n_extra_dev = halo_rows ? n_kept : nullptr; a.d = d;
  a.row_ptr = t_row_ptr; a.col_idx = t_col_idx; a.n_split = n_in;
  a.src0 = dA; a.src1 = nullptr; a.w_col = w_col; a.partials = partials;
  a.out0 = dH_in; a.out1 = dhalo; a.out_scale0 = row_scale; a.mask_src = mask_src;
  a.mask_scale = mask_scale;
  a.kept_ids = kept_ids; a.dis_halo = dis_halo; a.s_halo = s_halo;
  a.init = init; a.skip_self = skip_self;
  return launch_spmm(a, (int64_t)plan.n_seg + (halo_rows ? n_halo : 0), s);
}

// ------------------------------------------------------------------------------------------
// Static segmentation of a CSR pattern (set-up).
__global__ void __launch_bounds__(256)
seg_count_kernel(int32_t n_rows, const int32_t *__restrict__ row_ptr, int32_t *__restrict__ nseg) {
  const int v = blockIdx.x * 256 + threadIdx.x;
  if (v >= n_rows) return;
  const int len = row_ptr[v + 1] - row_ptr[v];
  nseg[v] = len <= kSegLen ? 1 : (len + kSegLen - 1) / kSegLen;
}

// which: 0 -> number of partial slots of the row (0 for single-segment rows), 1 -> multi flag
__global__ void __launch_bounds__(256)
seg_multi_kernel(int32_t n_rows, const int32_t *__restrict__ seg_ptr, int which, int32_t *__restrict__ out) {
  const int v = blockIdx.x * 256 + threadIdx.x;
  if (v >= n_rows) return;
  const int n = seg_ptr[v + 1] - seg_ptr[v];
  out[v] = n > 1 ? (which == 0 ? n : 1) : 0;
}

__global__ void __launch_bounds__(256)
seg_fill_kernel(int32_t n_rows, const int32_t *__restrict__ seg_ptr, const int32_t *__restrict__ mpos,
                int32_t *__restrict__ seg_row, int32_t *__restrict__ mrow) {
  const int v = blockIdx.x * 256 + threadIdx.x;
  if (v >= n_rows) return;
  const int s0 = seg_ptr[v], s1 = seg_ptr[v + 1];
  for (int s = s0; s < s1; ++s) seg_row[s] = v;
  if (s1 - s0 > 1) mrow[mpos[v]] = v;
}

hipError_t build_seg_plan(int32_t n_rows, int64_t nnz, const int32_t *row_ptr, SegPlan *plan, int32_t *tmp_a,
                          int32_t *tmp_b, int32_t *tile_sums, hipStream_t s) {
  const unsigned blocks = (unsigned)((n_rows + 255) / 256);
  seg_count_kernel<<<blocks, 256, 0, s>>>(n_rows, row_ptr, tmp_a);
  hipError_t e = scan_exclusive_i32(tmp_a, plan->seg_ptr, n_rows, nullptr, tile_sums, nullptr, 0, s);
  if (e != hipSuccess) return e;
  seg_multi_kernel<<<blocks, 256, 0, s>>>(n_rows, plan->seg_ptr, 0, tmp_a);
  e = scan_exclusive_i32(tmp_a, plan->part_ptr, n_rows, nullptr, tile_sums, nullptr, 0, s);
  if (e != hipSuccess) return e;
  seg_multi_kernel<<<blocks, 256, 0, s>>>(n_rows, plan->seg_ptr, 1, tmp_a);
  e = scan_exclusive_i32(tmp_a, tmp_b, n_rows, nullptr, tile_sums, nullptr, 0, s);
  if (e != hipSuccess) return e;
  seg_fill_kernel<<<blocks, 256, 0, s>>>(n_rows, plan->seg_ptr, tmp_b, plan->seg_row, plan->mrow);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  // the three totals size the launches: bring them to the host (set-up only)
  int32_t tot[3];
  e = hipMemcpyAsync(&tot[0], plan->seg_ptr + n_rows, 4, hipMemcpyDeviceToHost, s);
  if (e != hipSuccess) return e;
  e = hipMemcpyAsync(&tot[1], plan->part_ptr + n_rows, 4, hipMemcpyDeviceToHost, s);
  if (e != hipSuccess) return e;
  e = hipMemcpyAsync(&tot[2], tmp_b + n_rows, 4, hipMemcpyDeviceToHost, s);
  if (e != hipSuccess) return e;
  e = hipStreamSynchronize(s);
  if (e != hipSuccess) return e;
  plan->n_seg = tot[0];
  plan->n_part = tot[1];
  plan->n_multi = tot[2];
  plan->avg_len = n_rows > 0 ? (int32_t)(nnz / n_rows) : 0;
  return hipSuccess;
}

// ------------------------------------------------------------------------------------------
// Stand-in for "receive H_U" (Algorithm 1, feature exchange): gather the kept rows of the
// preloaded boundary features, scaled by S_uu = 1/p and by d~_u^-1/2 so that the aggregate
// adds them with weight one.
template <int VEC>
__global__ void __launch_bounds__(256)
halo_gather_kernel(const float *__restrict__ halo_h, const int32_t *__restrict__ kept_ids,
                   const int32_t *__restrict__ n_kept, const float *__restrict__ dis_halo,
                   float s_halo, int32_t d, float *__restrict__ Hu) {
  using V = typename Vec<VEC>::T;
  const int lane = lane_id();
  const int n = *n_kept;
  const int nvec = d / VEC;
  const int waves = gridDim.x * 4;
  for (int r = blockIdx.x * 4 + (threadIdx.x >> 6); r < n; r += waves) {
    const int b = kept_ids[r];
    const float sc = dis_halo ? s_halo * dis_halo[b] : s_halo;
    const V *src = reinterpret_cast<const V *>(halo_h + (size_t)b * d);
    V *dst = reinterpret_cast<V *>(Hu + (size_t)r * d);
    for (int iv = lane; iv < nvec; iv += kWave) {
      V x = src[iv];
      float *px = reinterpret_cast<float *>(&x);
#pragma unroll
      for (int i = 0; i < VEC; ++i) px[i] *= sc;
      dst[iv] = x;
    }
  }
}

hipError_t halo_gather(const float *halo_h, const int32_t *kept_ids, const int32_t *n_kept,
                       int32_t n_halo, const float *dis_halo, float s_halo, int32_t d, float *Hu,
                       hipStream_t s) {
  if (n_halo <= 0) return hipSuccess;
  int64_t blocks = ((int64_t)n_halo + 3) / 4;
  if (blocks > 8192) blocks = 8192;
  if (d % 4 == 0)
    halo_gather_kernel<4><<<(unsigned)blocks, 256, 0, s>>>(halo_h, kept_ids, n_kept, dis_halo, s_halo, d, Hu);
  else if (d % 2 == 0)
    halo_gather_kernel<2><<<(unsigned)blocks, 256, 0, s>>>(halo_h, kept_ids, n_kept, dis_halo, s_halo, d, Hu);
  else
    halo_gather_kernel<1><<<(unsigned)blocks, 256, 0, s>>>(halo_h, kept_ids, n_kept, dis_halo, s_halo, d, Hu);
  return hipGetLastError();
}

}  // namespace bns
