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

#include "spmm_device.hpp"

namespace bns {

// Measured on gfx950: the same code runs 3-6 % slower as soon as the wavefront needs more than 96
// scalar registers (seven 16-register granules instead of six), so the budget is pinned.
template <int VEC, int MAXCH, int LPR, bool NARROW = false>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_num_sgpr(96))) spmm_kernel(const SpmmArgs a) {
  using V = typename Vec<VEC>::T;
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
  const int n_units = a.multi_only ? a.plan.n_part : a.plan.n_seg + (a.n_extra_dev ? *a.n_extra_dev : 0);
  for (int unit = bid * 4 + (threadIdx.x >> 6); unit < n_units; unit += nblk * 4) {
  int row, seg = 0, nseg = 1;
  if (a.multi_only) {  // units are the partial-sum slots, i.e. the segments of the long rows
    row = a.plan.part_row[unit];
    seg = unit - a.plan.part_ptr[row];
    nseg = a.plan.seg_ptr[row + 1] - a.plan.seg_ptr[row];
  } else if (unit < a.plan.n_seg) {
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
  gather_segment<VEC, MAXCH, LPR>(a, row, e0, e1, d_off, nvec, acc);

  if (g != 0) {
    // only the first lane group holds the folded sums
  } else if (nseg == 1) {
    finish_row<VEC, MAXCH, NARROW>(a, row, sl, nvec, d_off, acc);
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
template <int VEC, int MAXCH, bool NARROW = false>
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
  finish_row<VEC, MAXCH, NARROW>(a, row, lane, nvec, 0, acc);
}

template <int VEC>
static hipError_t launch_spmm_vec(const SpmmArgs &a_in, int64_t max_units, hipStream_t s) {
  SpmmArgs a = a_in;
  a.n_slices = 1;
  a.d_slice = a.d;
  // Wide rows are cut into slices of 128 floats (64 where rows are long enough to keep a
  // wavefront busy with a quarter of its lanes per neighbour); measured on the five workloads,
  // narrower slices lose more to the repeated index walk than the L2 gains.
  if (VEC == 4 && !a.multi_only) {
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
  if (a.multi_only) blocks = (unsigned)((a.plan.n_part + 3) / 4);
  const unsigned cblocks = (unsigned)((a.plan.n_multi + 3) / 4);
  if (blocks == 0) return hipSuccess;
  if (a.n_slices > 1) {
    const unsigned per = 8 / a.n_slices;
    blocks = (blocks + per - 1) / per * 8;
  }
  if (a.d_store != a.d) {  // padded sources, dense narrower outputs: d < 128, four floats per lane
    if constexpr (VEC == 4) {
#define BNS_SPMM_NARROW(LPR) spmm_kernel<4, 1, LPR, true><<<blocks, 256, 0, s>>>(a)
      if (nvec <= 4) BNS_SPMM_NARROW(4);
      else if (nvec <= 8) BNS_SPMM_NARROW(8);
      else if (nvec <= 16) BNS_SPMM_NARROW(16);
      else BNS_SPMM_NARROW(32);
#undef BNS_SPMM_NARROW
      if (cblocks) spmm_combine_kernel<4, 1, true><<<cblocks, 256, 0, s>>>(a);
      return hipGetLastError();
    }
    return hipErrorInvalidValue;
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
  if (a.d_store != a.d && (a.d_store < 1 || a.d_store > a.d || a.d >= 128 || a.d % 4 != 0 || a.mask_src || a.init))
    return hipErrorInvalidValue;  // padded sources: narrow rows without mask or initial value only
  if (a.d % 4 == 0) return launch_spmm_vec<4>(a, max_units, s);
  if (a.d % 2 == 0) return launch_spmm_vec<2>(a, max_units, s);
  return launch_spmm_vec<1>(a, max_units, s);
}

hipError_t spmm_fwd(const SegPlan &plan, int32_t n_in, int32_t d, const int32_t *row_ptr,
                    const int32_t *col_idx, const float *w_col, const float *row_scale,
                    const float *H_in, const float *Hu, float *partials, float *A,
                    const SpmmRowPart &part, bool long_rows_only, bool relu, hipStream_t s, int32_t d_store) {
  SpmmArgs a = spmm_fwd_args(plan, n_in, d, row_ptr, col_idx, w_col, row_scale, H_in, Hu, partials, A, part);
  a.multi_only = long_rows_only;
  a.relu = relu;
  if (d_store > 0) a.d_store = d_store;
  return launch_spmm(a, plan.n_seg, s);
}

hipError_t spmm_bwd(const SegPlan &plan, int32_t n_in, int32_t n_halo, int32_t d,
                    const int32_t *t_row_ptr, const int32_t *t_col_idx, const int32_t *kept_ids,
                    const int32_t *n_kept, const float *w_col, const float *row_scale,
                    const float *dis_halo, float s_halo, const float *dA, const float *mask_src,
                    const float *init, bool skip_self, float *partials, float *dH_in, float *dhalo,
                    hipStream_t s, int32_t d_store) {
  SpmmArgs a{};
  const bool halo_rows = dhalo && n_halo > 0;
  a.plan = plan; a.n_extra_dev = halo_rows ? n_kept : nullptr; a.d = d; a.d_store = d_store > 0 ? d_store : d;
  a.row_ptr = t_row_ptr; a.col_idx = t_col_idx; a.n_split = n_in;
  a.src0 = dA; a.src1 = nullptr; a.w_col = w_col; a.partials = partials;
  a.out0 = dH_in; a.out1 = dhalo; a.out_scale0 = row_scale; a.mask_src = mask_src;
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
                const int32_t *__restrict__ part_ptr, int32_t *__restrict__ seg_row,
                int32_t *__restrict__ mrow, int32_t *__restrict__ part_row) {
  const int v = blockIdx.x * 256 + threadIdx.x;
  if (v >= n_rows) return;
  const int s0 = seg_ptr[v], s1 = seg_ptr[v + 1];
  for (int s = s0; s < s1; ++s) seg_row[s] = v;
  if (s1 - s0 > 1) {
    mrow[mpos[v]] = v;
    for (int s = 0; s < s1 - s0; ++s) part_row[part_ptr[v] + s] = v;
  }
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
  seg_fill_kernel<<<blocks, 256, 0, s>>>(n_rows, plan->seg_ptr, tmp_b, plan->part_ptr, plan->seg_row, plan->mrow,
                                         plan->part_row);
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
// Copy of a dense [n_rows, d] matrix with the rows padded by zeros to ld floats (ld a multiple of
// 4), so that an aggregate over a narrow odd width can gather with 16-byte loads.
__global__ void __launch_bounds__(256)
pad_rows_kernel(int64_t total, int32_t d, int32_t ld, const float *__restrict__ src, float *__restrict__ dst) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int64_t r = i / ld;
  const int c = (int)(i - r * ld);
  dst[i] = c < d ? src[r * d + c] : 0.f;
}

hipError_t pad_rows(int32_t n_rows, int32_t d, int32_t ld, const float *src, float *dst, hipStream_t s) {
  if (ld < d || d < 1) return hipErrorInvalidValue;
  const int64_t total = (int64_t)n_rows * ld;
  if (total == 0) return hipSuccess;
  pad_rows_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(total, d, ld, src, dst);
  return hipGetLastError();
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
  // one VEC-piece of one kept row per thread and step, consecutive threads on consecutive pieces
  // (a wavefront covers 64 / (d / VEC) rows); four independent pieces in flight per thread
  using V = typename Vec<VEC>::T;
  constexpr int UNR = 4;
  const unsigned nvec = (unsigned)(d / VEC);
  const long long total = (long long)*n_kept * nvec;
  const long long stride = (long long)gridDim.x * 256;
  const bool small = total + stride * UNR < 0x7fffffffLL;  // 32-bit division suffices
  for (long long t0 = (long long)blockIdx.x * 256 + threadIdx.x; t0 < total; t0 += stride * UNR) {
    int b[UNR];
    unsigned iv[UNR];
    long long t[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      t[u] = t0 + u * stride;
      const unsigned r = small ? (unsigned)t[u] / nvec : (unsigned)(t[u] / nvec);
      iv[u] = (unsigned)(t[u] - (long long)r * nvec);
      b[u] = t[u] < total ? kept_ids[r] : -1;
    }
    float sc[UNR];
    V x[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      sc[u] = (b[u] >= 0 && dis_halo) ? s_halo * dis_halo[b[u]] : s_halo;
      if (b[u] >= 0) x[u] = reinterpret_cast<const V *>(halo_h + (size_t)b[u] * d)[iv[u]];
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      if (b[u] < 0) continue;
      float *px = reinterpret_cast<float *>(&x[u]);
#pragma unroll
      for (int i = 0; i < VEC; ++i) px[i] *= sc[u];
      reinterpret_cast<V *>(Hu)[t[u]] = x[u];   // row r, piece iv: Hu is dense, so the piece index is t
    }
  }
}

__global__ void __launch_bounds__(256)
halo_records_kernel(const int32_t *__restrict__ kept_ids, const int32_t *__restrict__ n_kept,
                    const float *__restrict__ dis_halo, float s_halo, int2 *__restrict__ rec) {
  const int n = *n_kept;
  for (int r = blockIdx.x * 256 + threadIdx.x; r < n; r += gridDim.x * 256) {
    const int b = kept_ids[r];
    rec[r] = make_int2(b, __float_as_int(dis_halo ? s_halo * dis_halo[b] : s_halo));
  }
}

hipError_t halo_records(const int32_t *kept_ids, const int32_t *n_kept, int32_t n_halo, const float *dis_halo,
                        float s_halo, int2 *rec, hipStream_t s) {
  if (n_halo <= 0) return hipSuccess;
  const unsigned blocks = (unsigned)std::min<int64_t>(((int64_t)n_halo + 255) / 256, 2048);
  halo_records_kernel<<<blocks, 256, 0, s>>>(kept_ids, n_kept, dis_halo, s_halo, rec);
  return hipGetLastError();
}

hipError_t halo_gather(const float *halo_h, const int32_t *kept_ids, const int32_t *n_kept,
                       int32_t n_halo, const float *dis_halo, float s_halo, int32_t d, float *Hu,
                       hipStream_t s) {
  if (n_halo <= 0) return hipSuccess;
  const int vec = d % 4 == 0 ? 4 : d % 2 == 0 ? 2 : 1;
  int64_t blocks = ((int64_t)n_halo * (d / vec) + 1023) / 1024;  // sized for every boundary node kept
  if (blocks > 4096) blocks = 4096;
  if (d % 4 == 0)
    halo_gather_kernel<4><<<(unsigned)blocks, 256, 0, s>>>(halo_h, kept_ids, n_kept, dis_halo, s_halo, d, Hu);
  else if (d % 2 == 0)
    halo_gather_kernel<2><<<(unsigned)blocks, 256, 0, s>>>(halo_h, kept_ids, n_kept, dis_halo, s_halo, d, Hu);
  else
    halo_gather_kernel<1><<<(unsigned)blocks, 256, 0, s>>>(halo_h, kept_ids, n_kept, dis_halo, s_halo, d, Hu);
  return hipGetLastError();
}

}  // namespace bns
