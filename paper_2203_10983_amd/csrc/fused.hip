// Aggregate (Eq. 1) and update (Eq. 2) of one layer in one kernel: the GCN layer of Appendix A, or
// (SAGE) the mean-aggregator layer of Section 2, whose update [z | h] [W_n ; W_s] runs as two
// products from the same LDS tile: first the aggregated rows z times W_n, then, after the tile has
// been overwritten with the rows' own features h (one coalesced read), h times W_s into the same
// accumulators.
//
// The aggregate is bound by the rate at which the L2s pull neighbour rows from the fabric and
// leaves the matrix cores idle; the update of a 128-wide layer needs almost as much time for
// re-reading the aggregated rows as for its arithmetic.  Here a workgroup of 8 wavefronts
// aggregates a tile of 64 rows straight into LDS (each finished row also goes to global memory,
// because the weight gradient of the backward pass is A^T dZ), then multiplies the tile by W with
// v_mfma_f32_32x32x2_f32 while the other workgroups of the compute unit keep gathering.  W comes
// from L2 in 16-row pieces through a double-buffered LDS tile.
//
// Rows that the static plan cuts into several segments (longer than kSegLen entries) are not
// gathered here: a segmented pass has finished them before, and their row is read back.
#include "spmm_device.hpp"

namespace bns {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kFM = 64;           // rows per workgroup
constexpr int kFThreads = 512;    // 8 wavefronts: 2 (rows) x 4 (columns) MFMA tiles of 32 x 32
constexpr int kFLda = 129;        // odd row stride of the A tile: column reads hit 32 distinct banks
constexpr int kFBk = 16, kFBn = 128, kFLdb = kFBn + 4;

struct FusedArgs {
  SpmmArgs sp;
  const float *W;       // [d_in, d_out]; SAGE: [2 d_in, d_out], neighbour half first
  const float *H_self;  // SAGE: the layer's input [n_in, d_in] (the node's own features)
  float *H_out;         // [n_in, d_out]
  int32_t d_out;
  bool relu, vec_w;
  Dropout drop;
};

template <int LPR, bool SAGE>
__global__ void __launch_bounds__(kFThreads, 6) __attribute__((amdgpu_num_sgpr(96))) spmm_gemm_kernel(const FusedArgs f) {
  constexpr int VEC = 4;
  using V = typename Vec<VEC>::T;
  __shared__ float As[kFM * kFLda];
  __shared__ __attribute__((aligned(16))) float Bs[2][kFBk * kFLdb];
  const SpmmArgs &a = f.sp;
  const int lane = lane_id(), wid = threadIdx.x >> 6;
  const int g = lane / LPR, sl = lane % LPR;
  const int d = a.d, nvec = d / VEC;
  constexpr int k_pad = 128;  // depth of the tile product: d <= 128, zero-padded
  const int row0 = blockIdx.x * kFM;

  // ---- phase 0: the tile's row bounds into LDS (one coalesced read instead of a dependent chain
  // per row).  s_e0/s_e1: entries to gather; s_e1 < 0 marks a row finished by the segmented pass.
  __shared__ int s_e0[kFM], s_e1[kFM];
  __shared__ int next_row;
  if (threadIdx.x < kFM) {
    const int row = row0 + threadIdx.x;
    int e0 = 0, e1 = 0;
    if (row < a.n_split) {
      e0 = a.row_ptr[row];
      e1 = a.row_ptr[row + 1];
      if (a.row_skip) e0 += a.row_skip[row];
      if (a.row_take) e1 = e0 + a.row_take[row];
      if (a.plan.seg_ptr[row + 1] - a.plan.seg_ptr[row] > 1) e1 = -1;
    }
    s_e0[threadIdx.x] = e0;
    s_e1[threadIdx.x] = e1;
  }
  if (threadIdx.x == 0) next_row = 0;
  __syncthreads();

  // ---- phase 1: the wavefronts take rows from a shared counter and run them through a three-
  // stage pipeline, so that a row's index and weight reads are in flight while the previous rows
  // gather: stage A reads the column indices of row i+2, stage B the weights of row i+1, stage C
  // gathers row i (memory returns in issue order, so only the gather itself is waited for).
  auto grab = [&]() -> int {
    int r = 0;
    if (lane == 0) r = atomicAdd(&next_row, 1);
    return __builtin_amdgcn_readfirstlane(r);
  };
  auto first_cnt = [&](int lrow) -> int {  // entries of the row's first batch
    if (lrow >= kFM) return 0;
    const int e1 = s_e1[lrow];
    return e1 < 0 ? 0 : min(kWave, e1 - s_e0[lrow]);
  };
  auto stage_a = [&](int lrow) -> int {
    const int cnt = first_cnt(lrow);
    return lane < cnt ? a.col_idx[s_e0[lrow] + lane] : 0;
  };
  int j0 = grab();
  int c0 = stage_a(j0);
  int j1 = grab();
  int c1 = stage_a(j1);
  unsigned long long p0 = 0;
  float w0 = 0.f;
  if (lane < first_cnt(j0)) entry_source(a, row0 + j0, c0, 0, p0, w0);
  while (j0 < kFM) {
    const int j2 = grab();
    const int c2 = stage_a(j2);
    unsigned long long p1 = 0;
    float w1 = 0.f;
    if (lane < first_cnt(j1)) entry_source(a, row0 + j1, c1, 0, p1, w1);
    {  // stage C on row j0
      const int lrow = j0, row = row0 + lrow;
      float *lds_row = As + lrow * kFLda;
      const int e0 = s_e0[lrow], e1 = s_e1[lrow];
      if (row >= a.n_split) {  // past the last row: the tile is padded with zeros
        if (g == 0 && sl < nvec) {
#pragma unroll
          for (int i = 0; i < VEC; ++i) lds_row[sl * VEC + i] = 0.f;
        }
      } else if (e1 < 0) {  // finished by the segmented pass
        if (g == 0 && sl < nvec) {
          const V x = reinterpret_cast<const V *>(a.out0 + (size_t)row * d)[sl];
          const float *px = reinterpret_cast<const float *>(&x);
#pragma unroll
          for (int i = 0; i < VEC; ++i) lds_row[sl * VEC + i] = px[i];
        }
      } else {
        float acc[1][VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[0][i] = 0.f;
        gather_batch<VEC, 1, LPR>(p0, w0, min(kWave, e1 - e0), nvec, acc);
        for (int base = e0 + kWave; base < e1; base += kWave) {  // rows longer than one batch
          const int cnt = min(kWave, e1 - base);
          unsigned long long p_l = 0;
          float w_l = 0.f;
          if (lane < cnt) entry_source(a, row, a.col_idx[base + lane], 0, p_l, w_l);
          gather_batch<VEC, 1, LPR>(p_l, w_l, cnt, nvec, acc);
        }
        fold_groups<VEC, 1, LPR>(acc);
        if (g == 0) finish_row<VEC, 1>(a, row, sl, nvec, 0, acc, lds_row);
      }
      for (int k = d + lane; k < k_pad; k += kWave) lds_row[k] = 0.f;  // depth padding
    }
    j0 = j1; p0 = p1; w0 = w1;
    j1 = j2; c1 = c2;
  }
  // ---- phase 2: H_out tile = A tile x W ----------------------------------------------------------
  // W comes from L2 in 16-row pieces, each requested one step ahead (the first one before the
  // barrier that ends the gather) and passed through a double-buffered LDS tile.
  const int wm = (wid >> 2) * 32, wn = (wid & 3) * 32;
  const int l32 = lane & 31, lhi = lane >> 5;
  const int N = f.d_out;
  constexpr int nk = k_pad / kFBk;  // 8, an even number of steps
  const int t = threadIdx.x;
  const int bk = t >> 5, bq = (t & 31) * 4;  // this thread's piece of a W tile: row bk, columns bq..bq+3
  auto load_w_from = [&](const float *Wb, int n0, int k0) -> float4 {
    const int k = k0 + bk, c = n0 + bq;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (k < d && n0 < N) {
      const float *p = Wb + (size_t)k * N + c;
      if (f.vec_w && c + 3 < N) {
        v = *reinterpret_cast<const float4 *>(p);
      } else {
        if (c < N) v.x = p[0];
        if (c + 1 < N) v.y = p[1];
        if (c + 2 < N) v.z = p[2];
        if (c + 3 < N) v.w = p[3];
      }
    }
    return v;
  };
  auto load_w = [&](int n0, int k0) -> float4 { return load_w_from(f.W, n0, k0); };
  // C element of (lane, register r): row = 8*(r/4) + 4*(lane/32) + r%4, column = lane%32
  auto store_tile = [&](const floatx16 &acc, int n0) {
    const int col = n0 + wn + l32;
    if (col < N) {
#pragma unroll 1
      for (int q4 = 0; q4 < 4; ++q4) {
        const int row4 = row0 + wm + q4 * 8 + lhi * 4;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          const int row = row4 + rr;
          if (row < a.n_split) {
            float x = acc[q4 * 4 + rr];
            if (f.relu) {
              x = fmaxf(x, 0.f);
              if (f.drop.scale != 0.f) x = dropout_keeps(f.drop, row, col) ? x * f.drop.scale : 0.f;
            }
            __builtin_nontemporal_store(x, f.H_out + (size_t)row * N + col);  // streamed out, as the aggregate
          }
        }
      }
    }
  };
  float4 wv = load_w(0, 0);  // in flight across the barrier that ends the gather
  __syncthreads();
  if constexpr (SAGE) {
    // [z | h] [W_n ; W_s]: both operands pass through the one LDS tile, so the accumulators of every
    // column tile (at most two: d_out <= 256) stay live across the two products.
    floatx16 acc2[2];
#pragma unroll
    for (int tl = 0; tl < 2; ++tl)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc2[tl][i] = 0.f;
    const int ntile = (N + kFBn - 1) / kFBn;
#pragma unroll 1
    for (int op = 0; op < 2; ++op) {
      const float *Wop = f.W + (size_t)op * d * N;
      if (op == 1) {
        // every wavefront is past the barrier that ended the last step of z W_n: the tile is free.
        // Rows past the last one and the depth padding stay zero.
        for (int idx = t; idx < kFM * nvec; idx += kFThreads) {
          const int r = idx / nvec, c4 = idx - r * nvec;
          V x = V{};
          if (row0 + r < a.n_split) x = reinterpret_cast<const V *>(f.H_self + (size_t)(row0 + r) * d)[c4];
          const float *px = reinterpret_cast<const float *>(&x);
#pragma unroll
          for (int i = 0; i < VEC; ++i) As[r * kFLda + c4 * VEC + i] = px[i];
        }
      }
#pragma unroll
      for (int tl = 0; tl < 2; ++tl) {
        if (tl < ntile) {
          const int n0 = tl * kFBn;
          *reinterpret_cast<float4 *>(&Bs[0][bk * kFLdb + bq]) = wv;
          __syncthreads();  // also publishes the tile of own features written above
          const bool has_cols = n0 + wn < N;
#pragma unroll 1
          for (int kt = 0; kt < nk; ++kt) {
            const int buf = kt & 1;
            // the next piece: next depth step, else the first piece of the next column tile, else of W_s
            if (kt + 1 < nk) wv = load_w_from(Wop, n0, (kt + 1) * kFBk);
            else if (tl + 1 < ntile) wv = load_w_from(Wop, n0 + kFBn, 0);
            else if (op == 0) wv = load_w_from(f.W + (size_t)d * N, 0, 0);
            const float *as = As + (wm + l32) * kFLda + kt * kFBk + lhi;
            const float *bs = Bs[buf] + lhi * kFLdb + wn + l32;
            if (has_cols) {
#pragma unroll
              for (int kk = 0; kk < kFBk; kk += 2)
                acc2[tl] = __builtin_amdgcn_mfma_f32_32x32x2f32(as[kk], bs[kk * kFLdb], acc2[tl], 0, 0, 0);
            }
            if (kt + 1 < nk) *reinterpret_cast<float4 *>(&Bs[buf ^ 1][bk * kFLdb + bq]) = wv;
            __syncthreads();
          }
        }
      }
    }
    store_tile(acc2[0], 0);
    if (ntile > 1) store_tile(acc2[1], kFBn);
    return;
  }
  for (int n0 = 0; n0 < N; n0 += kFBn) {
    floatx16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
    *reinterpret_cast<float4 *>(&Bs[0][bk * kFLdb + bq]) = wv;
    __syncthreads();
    // a wavefront whose 32 columns all lie past the last one (the tail tile of a width such as
    // 172) still stages W and keeps the barriers, but issues no products
    const bool has_cols = n0 + wn < N;
#pragma unroll 1
    for (int kt = 0; kt < nk; ++kt) {
      const int buf = kt & 1;
      // request the next piece (next depth step, or the first one of the next column tile), issue
      // this step's products, and only then wait for the piece and stage it
      wv = kt + 1 < nk ? load_w(n0, (kt + 1) * kFBk) : load_w(n0 + kFBn, 0);
      const float *as = As + (wm + l32) * kFLda + kt * kFBk + lhi;
      const float *bs = Bs[buf] + lhi * kFLdb + wn + l32;
      if (has_cols) {
#pragma unroll
        for (int kk = 0; kk < kFBk; kk += 2)
          acc = __builtin_amdgcn_mfma_f32_32x32x2f32(as[kk], bs[kk * kFLdb], acc, 0, 0, 0);
      }
      if (kt + 1 < nk) *reinterpret_cast<float4 *>(&Bs[buf ^ 1][bk * kFLdb + bq]) = wv;
      __syncthreads();
    }
    store_tile(acc, n0);
  }
}

bool spmm_gemm_fwd_supported(int32_t d_in) { return d_in % 4 == 0 && d_in > 64 && d_in <= 128; }

bool spmm_gemm_fwd_concat_supported(int32_t d_in, int32_t d_out) {
  return spmm_gemm_fwd_supported(d_in) && d_out <= 2 * kFBn;
}

hipError_t spmm_gemm_fwd(const SegPlan &plan, int32_t n_in, int32_t d_in, int32_t d_out, const int32_t *row_ptr,
                         const int32_t *col_idx, const float *w_col, const float *row_scale,
                         const float *H_in, const float *Hu, float *partials, float *A,
                         const SpmmRowPart &part, const float *W, float *H_out, bool relu,
                         const Dropout &drop, hipStream_t s, bool concat_self) {
  if (!spmm_gemm_fwd_supported(d_in)) return hipErrorInvalidValue;
  if (concat_self && !spmm_gemm_fwd_concat_supported(d_in, d_out)) return hipErrorInvalidValue;
  if (n_in <= 0) return hipSuccess;
  FusedArgs f;
  f.sp = spmm_fwd_args(plan, n_in, d_in, row_ptr, col_idx, w_col, row_scale, H_in, Hu, partials, A, part);
  f.W = W;
  f.H_self = concat_self ? H_in : nullptr;
  f.H_out = H_out;
  f.d_out = d_out;
  f.relu = relu;
  f.vec_w = (d_out % 4 == 0) && (((uintptr_t)W & 15) == 0);
  f.drop = drop;
  const unsigned blocks = (unsigned)((n_in + kFM - 1) / kFM);
  if (concat_self) spmm_gemm_kernel<32, true><<<blocks, kFThreads, 0, s>>>(f);
  else spmm_gemm_kernel<32, false><<<blocks, kFThreads, 0, s>>>(f);
  return hipGetLastError();
}

}  // namespace bns
