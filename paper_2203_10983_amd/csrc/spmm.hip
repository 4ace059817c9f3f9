// Sparse aggregate (Eq. 1 in the sampled matrix form of Appendix A) and its transpose.
//
// One 64-lane wavefront owns one output row.  The lanes span the feature dimension with
// VEC-wide loads, so every neighbour row is read as one contiguous, coalesced segment.  When a
// feature row needs fewer than 64 lanes (LPR = lanes per row < 64) the wavefront walks 64/LPR
// neighbours at once and folds the partial sums at the end.  Column indices and their weights
// are fetched 64 at a time, one per lane, and handed to the loop by cross-lane reads, four
// neighbours in flight per step.  No atomics: the backward pass walks the transposed pattern,
// so every output element is produced by exactly one lane in a fixed order.
#include "device_utils.hpp"
#include "kernels.hpp"

namespace bns {

template <int VEC> struct Vec;
template <> struct Vec<1> { using T = float; };
template <> struct Vec<2> { using T = float2; };
template <> struct Vec<4> { using T = float4; };

template <int VEC>
__device__ __forceinline__ void vec_fma(float (&acc)[VEC], float w, const typename Vec<VEC>::T &v) {
  const float *p = reinterpret_cast<const float *>(&v);
#pragma unroll
  for (int i = 0; i < VEC; ++i) acc[i] = fmaf(w, p[i], acc[i]);
}

struct SpmmArgs {
  int32_t n_rows_static;       // rows when n_extra_dev == nullptr
  const int32_t *n_extra_dev;  // rows = n_rows_static + *n_extra_dev (transposed pass)
  int32_t d;
  const int32_t *row_ptr, *col_idx;
  int32_t n_split;             // columns < n_split read src0 (weight w_col[c]); others src1 (weight 1)
  const float *src0, *src1, *w_col;
  // output rows < n_split: out0 (scale out_scale0[row], optional mask); others: out1
  float *out0, *out1;
  const float *out_scale0;
  const float *mask_src;
  const int32_t *kept_ids;     // out1 row r is scaled by s_halo * dis_halo[kept_ids[r]]
  const float *dis_halo;
  float s_halo;
};

template <int VEC, int MAXCH, int LPR>
__global__ void __launch_bounds__(256) spmm_kernel(const SpmmArgs a) {
  using V = typename Vec<VEC>::T;
  constexpr int EP = kWave / LPR;  // neighbours walked at once
  constexpr int UNR = 4;
  const int lane = lane_id();
  const int g = lane / LPR, sl = lane % LPR;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int n_rows = a.n_rows_static + (a.n_extra_dev ? *a.n_extra_dev : 0);
  if (row >= n_rows) return;
  const int d = a.d;
  const int nvec = d / VEC;

  float acc[MAXCH][VEC];
#pragma unroll
  for (int c = 0; c < MAXCH; ++c)
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[c][i] = 0.f;

  const int e0 = a.row_ptr[row], e1 = a.row_ptr[row + 1];
  for (int base = e0; base < e1; base += kWave) {
    const int cnt = min(kWave, e1 - base);
    // one neighbour per lane: its feature-row address and weight
    unsigned long long p_l = 0;
    float w_l = 0.f;
    if (lane < cnt) {
      const int c = a.col_idx[base + lane];
      if (c < a.n_split) {
        p_l = (unsigned long long)(a.src0 + (size_t)c * d);
        w_l = a.w_col[c];
      } else {
        p_l = (unsigned long long)(a.src1 + (size_t)(c - a.n_split) * d);
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
    if (g != 0) return;
  }

  float scale;
  float *out;
  const float *mask = nullptr;
  if (row < a.n_split) {
    scale = a.out_scale0[row];
    out = a.out0 + (size_t)row * d;
    if (a.mask_src) mask = a.mask_src + (size_t)row * d;
  } else {
    if (a.out1 == nullptr) return;
    const int r = row - a.n_split;
    scale = a.s_halo * a.dis_halo[a.kept_ids[r]];
    out = a.out1 + (size_t)r * d;
  }
#pragma unroll
  for (int c = 0; c < MAXCH; ++c) {
    const int iv = c * kWave + sl;
    if (iv < nvec) {
      V o;
      float *po = reinterpret_cast<float *>(&o);
#pragma unroll
      for (int i = 0; i < VEC; ++i) po[i] = acc[c][i] * scale;
      if (mask) {
        const V m = reinterpret_cast<const V *>(mask)[iv];
        const float *pm = reinterpret_cast<const float *>(&m);
#pragma unroll
        for (int i = 0; i < VEC; ++i) po[i] = pm[i] > 0.f ? po[i] : 0.f;
      }
      reinterpret_cast<V *>(out)[iv] = o;
    }
  }
}

template <int VEC>
static hipError_t launch_spmm_vec(const SpmmArgs &a, int64_t max_rows, hipStream_t s) {
  const int nvec = a.d / VEC;
  const unsigned blocks = (unsigned)((max_rows + 3) / 4);
  if (blocks == 0) return hipSuccess;
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
  return hipGetLastError();
}

static hipError_t launch_spmm(const SpmmArgs &a, int64_t max_rows, hipStream_t s) {
  if (a.d % 4 == 0) return launch_spmm_vec<4>(a, max_rows, s);
  if (a.d % 2 == 0) return launch_spmm_vec<2>(a, max_rows, s);
  return launch_spmm_vec<1>(a, max_rows, s);
}

hipError_t spmm_fwd(int32_t n_in, int32_t d, const int32_t *row_ptr, const int32_t *col_idx,
                    const float *dis_in, const float *H_in, const float *Hu, float *A,
                    hipStream_t s) {
  SpmmArgs a{};
  a.n_rows_static = n_in; a.n_extra_dev = nullptr; a.d = d;
  a.row_ptr = row_ptr; a.col_idx = col_idx; a.n_split = n_in;
  a.src0 = H_in; a.src1 = Hu; a.w_col = dis_in;
  a.out0 = A; a.out1 = nullptr; a.out_scale0 = dis_in; a.mask_src = nullptr;
  a.kept_ids = nullptr; a.dis_halo = nullptr; a.s_halo = 0.f;
  return launch_spmm(a, n_in, s);
}

hipError_t spmm_bwd(int32_t n_in, int32_t n_halo, int32_t d, const int32_t *t_row_ptr,
                    const int32_t *t_col_idx, const int32_t *kept_ids, const int32_t *n_kept,
                    const float *dis_in, const float *dis_halo, float s_halo, const float *dA,
                    const float *mask_src, float *dH_in, float *dhalo, hipStream_t s) {
  SpmmArgs a{};
  a.n_rows_static = n_in; a.n_extra_dev = (dhalo && n_halo > 0) ? n_kept : nullptr; a.d = d;
  a.row_ptr = t_row_ptr; a.col_idx = t_col_idx; a.n_split = n_in;
  a.src0 = dA; a.src1 = nullptr; a.w_col = dis_in;
  a.out0 = dH_in; a.out1 = dhalo; a.out_scale0 = dis_in; a.mask_src = mask_src;
  a.kept_ids = kept_ids; a.dis_halo = dis_halo; a.s_halo = s_halo;
  const int64_t max_rows = (int64_t)n_in + ((dhalo && n_halo > 0) ? n_halo : 0);
  return launch_spmm(a, max_rows, s);
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
    const float sc = s_halo * dis_halo[b];
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
