// Dense update (Eq. 2) and its backward on the fp32 matrix cores (v_mfma_f32_32x32x2_f32).
//
// One kernel template covers the three products of a layer:
//   forward   H = A W            gemm_nn : A [M,K] k-contiguous,  B [K,N] n-contiguous
//   backward  dA = dZ W^T        gemm_nt : A [M,K] k-contiguous,  B [N,K] k-contiguous
//   backward  dW = A^T dZ        gemm_tn : A [K,M] m-contiguous,  B [K,N] n-contiguous, split K
// A 256-thread block (4 wavefronts, 2x2) owns a 128x128 tile of C; each wavefront owns 64x64 as
// 2x2 MFMA tiles of 32x32.  Operand tiles of depth 16 are staged through LDS in k-major order
// (As[k][m], Bs[k][n]) so that an MFMA operand read is one conflict-free row segment; the next
// tile is prefetched into registers while the current one is multiplied (double-buffered LDS,
// one barrier per step).  Split-K partial tiles are summed in a fixed order: no atomics.
#include "device_utils.hpp"
#include "kernels.hpp"

namespace bns {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BN = 128, BK = 16;
constexpr int LDS_LD = BM + 4;  // row stride of a staged tile in floats (keeps 16-byte alignment)
constexpr int kGemmThreads = 256;

// Tile of an operand stored [rows][K] (k-contiguous): 128 rows x 16 k, as 2 x float4 per thread.
struct FragK { float4 v[2]; };
// Tile of an operand stored [K][cols] (contiguous along the tile's 128 columns).
struct FragN { float4 v[2]; };

__device__ __forceinline__ float4 load4_guarded(const float *p, bool vec_ok, int valid) {
  // valid = number of leading elements (0..4) that are in range
  if (vec_ok && valid == 4) return *reinterpret_cast<const float4 *>(p);
  float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
  if (valid > 0) r.x = p[0];
  if (valid > 1) r.y = p[1];
  if (valid > 2) r.z = p[2];
  if (valid > 3) r.w = p[3];
  return r;
}

__device__ __forceinline__ int clamp04(int x) { return x < 0 ? 0 : (x > 4 ? 4 : x); }

// rows: row0.. of an operand [R][ld] (k-contiguous); k range [k0, k0+16) limited by k_end
__device__ __forceinline__ void load_kcontig(FragK &f, const float *__restrict__ base, int ld,
                                             int row0, int n_rows, int k0, int k_end, bool vec_ok) {
  const int t = threadIdx.x;
  const int kq = (t & 3) * 4;
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int r = row0 + (t >> 2) + p * 64;
    const int valid = r < n_rows ? clamp04(k_end - (k0 + kq)) : 0;
    f.v[p] = load4_guarded(base + (size_t)r * ld + k0 + kq, vec_ok, valid);
  }
}
__device__ __forceinline__ void store_kcontig(const FragK &f, float *__restrict__ tile) {
  const int t = threadIdx.x;
  const int kq = (t & 3) * 4;
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int r = (t >> 2) + p * 64;
    tile[(kq + 0) * LDS_LD + r] = f.v[p].x;
    tile[(kq + 1) * LDS_LD + r] = f.v[p].y;
    tile[(kq + 2) * LDS_LD + r] = f.v[p].z;
    tile[(kq + 3) * LDS_LD + r] = f.v[p].w;
  }
}

// operand [K][ld] with the tile's 128 columns starting at col0
__device__ __forceinline__ void load_ncontig(FragN &f, const float *__restrict__ base, int ld,
                                             int col0, int n_cols, int k0, int k_end, bool vec_ok) {
  const int t = threadIdx.x;
  const int cq = (t & 31) * 4;
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int k = k0 + (t >> 5) + p * 8;
    const int valid = k < k_end ? clamp04(n_cols - (col0 + cq)) : 0;
    f.v[p] = load4_guarded(base + (size_t)k * ld + col0 + cq, vec_ok, valid);
  }
}
__device__ __forceinline__ void store_ncontig(const FragN &f, float *__restrict__ tile) {
  const int t = threadIdx.x;
  const int cq = (t & 31) * 4;
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int k = (t >> 5) + p * 8;
    *reinterpret_cast<float4 *>(&tile[k * LDS_LD + cq]) = f.v[p];
  }
}

template <bool A_KCONTIG, bool B_KCONTIG, bool RELU>
__global__ void __launch_bounds__(kGemmThreads)
gemm_kernel(int M, int N, int K, const float *__restrict__ A, int lda, const float *__restrict__ B,
            int ldb, float *__restrict__ C, int ldc, int k_chunk, bool vec_a, bool vec_b) {
  __shared__ __attribute__((aligned(16))) float As[2][BK * LDS_LD];
  __shared__ __attribute__((aligned(16))) float Bs[2][BK * LDS_LD];

  const int tiles_n = (N + BN - 1) / BN;
  const int tm = blockIdx.x / tiles_n, tn = blockIdx.x % tiles_n;
  const int bm0 = tm * BM, bn0 = tn * BN;
  const int k_begin = blockIdx.y * k_chunk;
  const int k_end = min(K, k_begin + k_chunk);
  C += (size_t)blockIdx.y * M * ldc;  // split-K: one partial matrix per split

  const int lane = lane_id(), wid = threadIdx.x >> 6;
  const int wm = (wid >> 1) * 64, wn = (wid & 1) * 64;
  const int l32 = lane & 31, lhi = lane >> 5;

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  using FA = typename std::conditional<A_KCONTIG, FragK, FragN>::type;
  using FB = typename std::conditional<B_KCONTIG, FragK, FragN>::type;
  FA fa;
  FB fb;
  auto load_tiles = [&](int k0) {
    if constexpr (A_KCONTIG) load_kcontig(fa, A, lda, bm0, M, k0, k_end, vec_a);
    else load_ncontig(fa, A, lda, bm0, M, k0, k_end, vec_a);
    if constexpr (B_KCONTIG) load_kcontig(fb, B, ldb, bn0, N, k0, k_end, vec_b);
    else load_ncontig(fb, B, ldb, bn0, N, k0, k_end, vec_b);
  };
  auto store_tiles = [&](int buf) {
    if constexpr (A_KCONTIG) store_kcontig(fa, As[buf]); else store_ncontig(fa, As[buf]);
    if constexpr (B_KCONTIG) store_kcontig(fb, Bs[buf]); else store_ncontig(fb, Bs[buf]);
  };

  const int nk = (k_end - k_begin + BK - 1) / BK;
  if (nk > 0) {
    load_tiles(k_begin);
    store_tiles(0);
  }
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) load_tiles(k_begin + (kt + 1) * BK);
    const float *as = As[buf] + wm + l32;
    const float *bs = Bs[buf] + wn + l32;
#pragma unroll
    for (int kk = 0; kk < BK; kk += 2) {
      const int krow = (kk + lhi) * LDS_LD;
      const float a0 = as[krow], a1 = as[krow + 32];
      const float b0 = bs[krow], b1 = bs[krow + 32];
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
    }
    if (kt + 1 < nk) store_tiles(buf ^ 1);
    __syncthreads();
  }

  // C tile element held by (lane, register r): row = 8*(r/4) + 4*(lane/32) + r%4, col = lane%32
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int col = bn0 + wn + j * 32 + l32;
      if (col >= N) continue;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = bm0 + wm + i * 32 + (r >> 2) * 8 + lhi * 4 + (r & 3);
        if (row < M) {
          float x = acc[i][j][r];
          if (RELU) x = fmaxf(x, 0.f);
          C[(size_t)row * ldc + col] = x;
        }
      }
    }
}

static inline bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }

hipError_t gemm_nn(int32_t M, int32_t N, int32_t K, const float *A, const float *B, float *C,
                   bool relu, hipStream_t s) {
  const unsigned tiles = (unsigned)(((M + BM - 1) / BM) * ((N + BN - 1) / BN));
  if (tiles == 0) return hipSuccess;
  const bool va = (K % 4 == 0) && aligned16(A), vb = (N % 4 == 0) && aligned16(B);
  if (relu)
    gemm_kernel<true, false, true><<<dim3(tiles, 1), kGemmThreads, 0, s>>>(M, N, K, A, K, B, N, C, N, K, va, vb);
  else
    gemm_kernel<true, false, false><<<dim3(tiles, 1), kGemmThreads, 0, s>>>(M, N, K, A, K, B, N, C, N, K, va, vb);
  return hipGetLastError();
}

hipError_t gemm_nt(int32_t M, int32_t N, int32_t K, const float *A, const float *B, float *C,
                   hipStream_t s) {
  const unsigned tiles = (unsigned)(((M + BM - 1) / BM) * ((N + BN - 1) / BN));
  if (tiles == 0) return hipSuccess;
  const bool va = (K % 4 == 0) && aligned16(A), vb = (K % 4 == 0) && aligned16(B);
  gemm_kernel<true, true, false><<<dim3(tiles, 1), kGemmThreads, 0, s>>>(M, N, K, A, K, B, K, C, N, K, va, vb);
  return hipGetLastError();
}

// ---- split-K -----------------------------------------------------------------------------------
constexpr int kSplitTargetBlocks = 768;
constexpr int kReduceGroup = 16;

static inline int splitk_chunk(int32_t M, int32_t N, int32_t K, int *splits_out) {
  const int tiles = ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
  int splits = (kSplitTargetBlocks + tiles - 1) / tiles;
  const int max_splits = (K + 4 * BK - 1) / (4 * BK);  // at least 64 rows of K per split
  if (splits > max_splits) splits = max_splits;
  if (splits < 1) splits = 1;
  int chunk = (K + splits - 1) / splits;
  chunk = ((chunk + BK - 1) / BK) * BK;
  splits = (K + chunk - 1) / chunk;
  if (splits < 1) splits = 1;
  *splits_out = splits;
  return chunk;
}

int32_t splitk_splits(int32_t M, int32_t N, int32_t K) {
  int s;
  splitk_chunk(M, N, K, &s);
  // first-level partials plus the second-level buffer of the grouped reduction
  return s + (s + kReduceGroup - 1) / kReduceGroup;
}

// out[g][i] = sum over the splits z of group g (in ascending z) of in[z][i]
__global__ void __launch_bounds__(256)
splitk_reduce_kernel(const float *__restrict__ in, float *__restrict__ out, int64_t mn, int splits) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= mn) return;
  const int z0 = blockIdx.y * kReduceGroup;
  const int z1 = min(splits, z0 + kReduceGroup);
  float sum = 0.f;
  for (int z = z0; z < z1; ++z) sum += in[(size_t)z * mn + i];
  out[(size_t)blockIdx.y * mn + i] = sum;
}

hipError_t gemm_tn_splitk(int32_t M, int32_t N, int32_t K, const float *A, const float *B,
                          float *C, float *partials, hipStream_t s) {
  const unsigned tiles = (unsigned)(((M + BM - 1) / BM) * ((N + BN - 1) / BN));
  if (tiles == 0) return hipSuccess;
  int splits;
  const int chunk = splitk_chunk(M, N, K, &splits);
  const bool va = (M % 4 == 0) && aligned16(A), vb = (N % 4 == 0) && aligned16(B);
  const int64_t mn = (int64_t)M * N;
  float *dst = splits == 1 ? C : partials;
  gemm_kernel<false, false, false><<<dim3(tiles, splits), kGemmThreads, 0, s>>>(
      M, N, K, A, M, B, N, dst, N, chunk, va, vb);
  // grouped, fixed-order reduction: partials -> level 2 -> ... -> C
  float *cur = partials;
  float *nxt = partials + (size_t)splits * mn;
  int n = splits;
  while (n > 1) {
    const int groups = (n + kReduceGroup - 1) / kReduceGroup;
    float *out = groups == 1 ? C : nxt;
    splitk_reduce_kernel<<<dim3((unsigned)((mn + 255) / 256), groups), 256, 0, s>>>(cur, out, mn, n);
    float *t = cur; cur = nxt; nxt = t;   // ping-pong (level >= 3 reuses the first buffer)
    n = groups;
  }
  return hipGetLastError();
}

}  // namespace bns
