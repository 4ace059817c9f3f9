// Dense update (Eq. 2) and its backward on the fp32 matrix cores (v_mfma_f32_32x32x2_f32).
//
// One kernel template covers the three products of a layer:
//   forward   H = A W            gemm_nn : A [M,K] k-contiguous,  B [K,N] n-contiguous
//   backward  dA = dZ W^T        gemm_nt : A [M,K] k-contiguous,  B [N,K] k-contiguous
//   backward  dW = A^T dZ        gemm_tn : A [K,M] m-contiguous,  B [K,N] n-contiguous, split K
// A block owns a 128 x BN tile of C.  BN = 128 with a k-contiguous A (forward product, dZ W^T): 8
// wavefronts (2 x 4), each 64 x 32 = two 32x32 accumulators; BN = 128 with an m-contiguous A (the
// split-K weight gradient): 4 wavefronts (2 x 2), each 64 x 64; BN = 64 (chosen when it wastes
// fewer padded columns, e.g. N = 172, 47, 41): 4 wavefronts (4 x 1), each 32 x 64.  Measured on
// gfx950: the matrix pipe itself issues at 98 % of its peak whatever the number of wavefronts per
// SIMD and of accumulators per wavefront (bns_probe_mfma), so a tile shape is judged by how well it
// hides operand staging and barriers: stand-alone the 8-wavefront tile (six to eight wavefronts per
// SIMD instead of four) is 10 - 26 % faster than the 4-wavefront one, inside a training step 3 - 8 %
// (the weight gradient, which streams both operands, lost 1 - 3 % and keeps four wavefronts).
// Operand tiles of depth 16 are staged through LDS
// in k-major order (As[k][m], Bs[k][n]) so that an MFMA operand read is one conflict-free row
// segment; the next tile is prefetched into registers while the current one is multiplied
// (double-buffered LDS, one barrier per step).  Split-K partial tiles are summed in a fixed
// order: no atomics.
#include <type_traits>

#include "device_utils.hpp"
#include "kernels.hpp"

namespace bns {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BK = 16;
constexpr int gemm_threads(int bn, bool a_kcontig) { return (bn == 128 && a_kcontig) ? 512 : 256; }

// Tile of an operand stored [rows][K] (k-contiguous): ROWS rows x 16 k, one float4 per thread and pass.
template <int ROWS, int NT> struct FragK { float4 v[ROWS * 4 / NT]; };
// Tile of an operand stored [K][cols] (contiguous along the tile's COLS columns).
template <int COLS, int NT> struct FragN { float4 v[BK * COLS / 4 / NT]; };

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

// rows row0.. of an operand [R][ld] (k-contiguous); k range [k0, k0+16) limited by k_end
template <int ROWS, int NT>
__device__ __forceinline__ void load_kcontig(FragK<ROWS, NT> &f, const float *__restrict__ base, int ld,
                                             int row0, int n_rows, int k0, int k_end, bool vec_ok) {
  constexpr int PASSES = ROWS * 4 / NT, RPP = NT / 4;  // rows per pass
  const int t = threadIdx.x;
  const int kq = (t & 3) * 4;
  if (vec_ok && row0 + ROWS <= n_rows && k0 + BK <= k_end) {  // whole tile in range (uniform over the block)
#pragma unroll
    for (int p = 0; p < PASSES; ++p)
      f.v[p] = *reinterpret_cast<const float4 *>(base + (size_t)(row0 + (t >> 2) + p * RPP) * ld + k0 + kq);
    return;
  }
#pragma unroll
  for (int p = 0; p < PASSES; ++p) {
    const int r = row0 + (t >> 2) + p * RPP;
    const int valid = r < n_rows ? clamp04(k_end - (k0 + kq)) : 0;
    f.v[p] = load4_guarded(base + (size_t)r * ld + k0 + kq, vec_ok, valid);
  }
}
template <int ROWS, int NT>
__device__ __forceinline__ void store_kcontig(const FragK<ROWS, NT> &f, float *__restrict__ tile) {
  constexpr int LD = ROWS + 4;
  constexpr int PASSES = ROWS * 4 / NT, RPP = NT / 4;
  const int t = threadIdx.x;
  const int kq = (t & 3) * 4;
#pragma unroll
  for (int p = 0; p < PASSES; ++p) {
    const int r = (t >> 2) + p * RPP;
    tile[(kq + 0) * LD + r] = f.v[p].x;
    tile[(kq + 1) * LD + r] = f.v[p].y;
    tile[(kq + 2) * LD + r] = f.v[p].z;
    tile[(kq + 3) * LD + r] = f.v[p].w;
  }
}

// operand [K][ld] with the tile's COLS columns starting at col0
template <int COLS, int NT>
__device__ __forceinline__ void load_ncontig(FragN<COLS, NT> &f, const float *__restrict__ base, int ld,
                                             int col0, int n_cols, int k0, int k_end, bool vec_ok) {
  constexpr int TPR = COLS / 4;              // threads per k-row
  constexpr int KPP = NT / TPR;              // k-rows per pass
  const int t = threadIdx.x;
  const int cq = (t % TPR) * 4;
  if (vec_ok && col0 + COLS <= n_cols && k0 + BK <= k_end) {  // whole tile in range (uniform over the block)
#pragma unroll
    for (int p = 0; p < BK / KPP; ++p)
      f.v[p] = *reinterpret_cast<const float4 *>(base + (size_t)(k0 + t / TPR + p * KPP) * ld + col0 + cq);
    return;
  }
#pragma unroll
  for (int p = 0; p < BK / KPP; ++p) {
    const int k = k0 + t / TPR + p * KPP;
    const int valid = k < k_end ? clamp04(n_cols - (col0 + cq)) : 0;
    f.v[p] = load4_guarded(base + (size_t)k * ld + col0 + cq, vec_ok, valid);
  }
}
template <int COLS, int LD, int NT>
__device__ __forceinline__ void store_ncontig(const FragN<COLS, NT> &f, float *__restrict__ tile) {
  constexpr int TPR = COLS / 4;
  constexpr int KPP = NT / TPR;
  const int t = threadIdx.x;
  const int cq = (t % TPR) * 4;
#pragma unroll
  for (int p = 0; p < BK / KPP; ++p) {
    const int k = t / TPR + p * KPP;
    *reinterpret_cast<float4 *>(&tile[k * LD + cq]) = f.v[p];
  }
}

// EPI: 0 = store alpha * product, 1 = ReLU, 2 = zero where mask_src <= 0, alpha * product elsewhere
// (ReLU/dropout mask of the backward pass), 3 = add to C, 4 = add to C then ReLU.  With EPI 1 or 4 and drop.scale != 0
// the ReLU output goes through dropout (one counter-based draw per element).
// m_dev (nullable): the row count lives on the device (*m_dev <= M); tiles past it do nothing.
// k_dev (nullable): the depth lives on the device (*k_dev <= K); steps past it contribute nothing.
// A2 (nullable, k-contiguous A only): the operand is the concatenation [A | A2] along the depth,
// both with row stride lda = a_split (a multiple of 16); for the m-contiguous A of the transposed
// product it is the concatenation along M (a_split a multiple of 128).  C2 (nullable): the result is the pair
// [C | C2] split at column c_split (a multiple of the column tile), both with row stride ldc.
template <int BN, bool A_KCONTIG, bool B_KCONTIG, int EPI>
// The 8-wavefront tile is held to 64 registers, so that four workgroups (eight wavefronts per SIMD) fit a
// compute unit: 1 - 2 % on the 512-wide products over three workgroups at 68 registers.
__global__ void __launch_bounds__(gemm_threads(BN, A_KCONTIG), (BN == 128 && A_KCONTIG) ? 8 : 4)
gemm_kernel(int M, int N, int K, const float *__restrict__ A, int lda, const float *__restrict__ B,
            int ldb, float *__restrict__ C, int ldc, int k_chunk, bool vec_a, bool vec_b,
            const float *__restrict__ mask_src, float alpha, const int *__restrict__ m_dev,
            const int *__restrict__ k_dev, const Dropout drop, const float *__restrict__ A2, int a_split,
            float *__restrict__ C2, int c_split) {
  // Every tile is staged through registers.  (Filling the W tile of the forward product straight
  // into LDS with global_load_lds paid with four wavefronts per block, costs 3 % with eight; doing
  // it for both tiles of the transposed product was 25 % slower.)
  constexpr int LDA = BM + 4, LDB = BN + 4;
  constexpr int NT = gemm_threads(BN, A_KCONTIG);
  constexpr bool kEight = NT == 512;
  constexpr int TI = BN == 128 ? 2 : 1, TJ = kEight ? 1 : 2;  // 32 x 32 MFMA tiles per wavefront: TI x TJ
  const int m_full = M;
  if (m_dev) M = min(M, *m_dev);
  if (k_dev) K = min(K, *k_dev);  // the depth lives on the device (kept boundary rows)
  __shared__ __attribute__((aligned(16))) float As[2][BK * LDA];
  __shared__ __attribute__((aligned(16))) float Bs[2][BK * LDB];

  const int tiles_n = (N + BN - 1) / BN;
  const int tm = blockIdx.x / tiles_n, tn = blockIdx.x % tiles_n;
  const int bm0 = tm * BM, bn0 = tn * BN;
  if (bm0 >= M) return;
  const int k_begin = blockIdx.y * k_chunk;
  const int k_end = min(K, k_begin + k_chunk);
  C += (size_t)blockIdx.y * m_full * ldc;  // split-K: one partial matrix per split

  const int lane = lane_id(), wid = threadIdx.x >> 6;
  const int wm = kEight ? (wid >> 2) * 64 : BN == 128 ? (wid >> 1) * 64 : wid * 32;
  const int wn = kEight ? (wid & 3) * 32 : BN == 128 ? (wid & 1) * 64 : 0;
  const int l32 = lane & 31, lhi = lane >> 5;

  floatx16 acc[TI][TJ];
#pragma unroll
  for (int i = 0; i < TI; ++i)
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  using FA = typename std::conditional<A_KCONTIG, FragK<BM, NT>, FragN<BM, NT>>::type;
  using FB = typename std::conditional<B_KCONTIG, FragK<BN, NT>, FragN<BN, NT>>::type;
  FA fa;
  FB fb;
  auto load_tiles = [&](int k0) {
    if constexpr (A_KCONTIG) {
      const float *Ab = A;
      int k0a = k0, kea = k_end;
      if (A2) {  // a depth tile never straddles the seam: a_split is a multiple of BK
        if (k0 >= a_split) { Ab = A2; k0a = k0 - a_split; kea = k_end - a_split; }
        else kea = min(k_end, a_split);
      }
      load_kcontig<BM, NT>(fa, Ab, lda, bm0, M, k0a, kea, vec_a);
    } else {
      // [A | A2] along the columns of the m-contiguous operand: a row tile lies in one of them
      const float *Ab = (A2 && bm0 >= a_split) ? A2 : A;
      const int c0 = (A2 && bm0 >= a_split) ? bm0 - a_split : bm0;
      const int nc = A2 ? a_split : M;
      load_ncontig<BM, NT>(fa, Ab, lda, c0, nc, k0, k_end, vec_a);
    }
    if constexpr (B_KCONTIG) {
      load_kcontig<BN, NT>(fb, B, ldb, bn0, N, k0, k_end, vec_b);
    } else {
      load_ncontig<BN, NT>(fb, B, ldb, bn0, N, k0, k_end, vec_b);
    }
  };
  auto store_tiles = [&](int buf) {
    if constexpr (A_KCONTIG) store_kcontig<BM, NT>(fa, As[buf]);
    else store_ncontig<BM, LDA, NT>(fa, As[buf]);
    if constexpr (B_KCONTIG) store_kcontig<BN, NT>(fb, Bs[buf]);
    else store_ncontig<BN, LDB, NT>(fb, Bs[buf]);
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
      float a[TI], b[TJ];
#pragma unroll
      for (int i = 0; i < TI; ++i) a[i] = as[(kk + lhi) * LDA + i * 32];
#pragma unroll
      for (int j = 0; j < TJ; ++j) b[j] = bs[(kk + lhi) * LDB + j * 32];
#pragma unroll
      for (int i = 0; i < TI; ++i)
#pragma unroll
        for (int j = 0; j < TJ; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) store_tiles(buf ^ 1);
    __syncthreads();
  }

  // C tile element held by (lane, register r): row = 8*(r/4) + 4*(lane/32) + r%4, col = lane%32
#pragma unroll
  for (int i = 0; i < TI; ++i)
#pragma unroll
    for (int j = 0; j < TJ; ++j) {
      int col = bn0 + wn + j * 32 + l32;
      // a result with padded rows (ldc > N, plain store only): columns N..ldc-1 are cleared
      const bool pad_col = col >= N;
      if (pad_col && !(EPI == 0 && C2 == nullptr && col < ldc)) continue;
      float *Cd = C;
      if (C2 && col >= c_split) { Cd = C2; col -= c_split; }  // column tiles never straddle c_split
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int row4 = bm0 + wm + i * 32 + q4 * 8 + lhi * 4;  // a multiple of 4
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          const int row = row4 + rr;
          if (row < M) {
            float x = acc[i][j][q4 * 4 + rr];
            if (EPI == 3 || EPI == 4) x += Cd[(size_t)row * ldc + col];
            if (EPI == 1 || EPI == 4) {
              x = fmaxf(x, 0.f);
              if (drop.scale != 0.f) x = dropout_keeps(drop, row, col) ? x * drop.scale : 0.f;
            }
            if (EPI == 2) x = mask_src[(size_t)row * ldc + col] > 0.f ? x * alpha : 0.f;
            if (EPI == 0) x = pad_col ? 0.f : x * alpha;
            Cd[(size_t)row * ldc + col] = x;
          }
        }
      }
    }
}

static inline bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }

// Column-tile width: the one that pads N to fewer columns (ties go to the wider tile).
static inline int pick_bn(int N) {
  const int pad128 = (N + 127) / 128 * 128, pad64 = (N + 63) / 64 * 64;
  return pad64 < pad128 ? 64 : 128;
}
static inline unsigned n_tiles(int M, int N, int bn) {
  return (unsigned)(((M + BM - 1) / BM) * ((N + bn - 1) / bn));
}

#define BNS_GEMM_LAUNCH(AK, BK_, EPI, grid, ...)                                                 \
  do {                                                                                           \
    if (bn == 64) gemm_kernel<64, AK, BK_, EPI><<<grid, gemm_threads(64, AK), 0, s>>>(__VA_ARGS__);  \
    else gemm_kernel<128, AK, BK_, EPI><<<grid, gemm_threads(128, AK), 0, s>>>(__VA_ARGS__);         \
  } while (0)

hipError_t gemm_nn(int32_t M, int32_t N, int32_t K, const float *A, const float *B, float *C,
                   bool relu, bool accumulate, const Dropout &drop, const int32_t *m_dev, hipStream_t s,
                   int32_t ldc) {
  if (ldc == 0) ldc = N;
  if (ldc < N) return hipErrorInvalidValue;
  const int bn = pick_bn(N);
  const unsigned tiles = n_tiles(M, N, bn);
  if (tiles == 0) return hipSuccess;
  const bool va = (K % 4 == 0) && aligned16(A), vb = (N % 4 == 0) && aligned16(B);
  const dim3 grid(tiles, 1);
  if (accumulate && relu) BNS_GEMM_LAUNCH(true, false, 4, grid, M, N, K, A, K, B, N, C, ldc, K, va, vb, nullptr, 1.f, m_dev, nullptr, drop, nullptr, 0, nullptr, 0);
  else if (accumulate) BNS_GEMM_LAUNCH(true, false, 3, grid, M, N, K, A, K, B, N, C, ldc, K, va, vb, nullptr, 1.f, m_dev, nullptr, drop, nullptr, 0, nullptr, 0);
  else if (relu) BNS_GEMM_LAUNCH(true, false, 1, grid, M, N, K, A, K, B, N, C, ldc, K, va, vb, nullptr, 1.f, m_dev, nullptr, drop, nullptr, 0, nullptr, 0);
  else BNS_GEMM_LAUNCH(true, false, 0, grid, M, N, K, A, K, B, N, C, ldc, K, va, vb, nullptr, 1.f, m_dev, nullptr, drop, nullptr, 0, nullptr, 0);
  return hipGetLastError();
}

hipError_t gemm_nn_concat(int32_t M, int32_t N, int32_t K_half, const float *A1, const float *A2,
                          const float *B, float *C, bool relu, const Dropout &drop, hipStream_t s) {
  if (K_half % BK != 0) return hipErrorInvalidValue;
  const int bn = pick_bn(N);
  const unsigned tiles = n_tiles(M, N, bn);
  if (tiles == 0) return hipSuccess;
  const int K = 2 * K_half;
  const bool va = (K_half % 4 == 0) && aligned16(A1) && aligned16(A2), vb = (N % 4 == 0) && aligned16(B);
  const dim3 grid(tiles, 1);
  if (relu) BNS_GEMM_LAUNCH(true, false, 1, grid, M, N, K, A1, K_half, B, N, C, N, K, va, vb, nullptr, 1.f, nullptr, nullptr, drop, A2, K_half, nullptr, 0);
  else BNS_GEMM_LAUNCH(true, false, 0, grid, M, N, K, A1, K_half, B, N, C, N, K, va, vb, nullptr, 1.f, nullptr, nullptr, drop, A2, K_half, nullptr, 0);
  return hipGetLastError();
}

bool gemm_nt_pair_supported(int32_t N_half) { return N_half % 64 == 0; }

hipError_t gemm_nt_pair(int32_t M, int32_t N_half, int32_t K, const float *A, const float *B, float *C1,
                        float *C2, float alpha, hipStream_t s) {
  if (!gemm_nt_pair_supported(N_half)) return hipErrorInvalidValue;
  const int N = 2 * N_half;
  const int bn = N_half % 128 == 0 ? 128 : 64;  // a column tile must not straddle the two results
  const unsigned tiles = n_tiles(M, N, bn);
  if (tiles == 0) return hipSuccess;
  const bool va = (K % 4 == 0) && aligned16(A), vb = (K % 4 == 0) && aligned16(B);
  const dim3 grid(tiles, 1);
  BNS_GEMM_LAUNCH(true, true, 0, grid, M, N, K, A, K, B, K, C1, N_half, K, va, vb, nullptr, alpha, nullptr, nullptr, Dropout{}, nullptr, 0, C2, N_half);
  return hipGetLastError();
}

hipError_t gemm_nt(int32_t M, int32_t N, int32_t K, const float *A, const float *B, float *C,
                   const float *mask_src, float alpha, const int32_t *m_dev, hipStream_t s) {
  const int bn = pick_bn(N);
  const unsigned tiles = n_tiles(M, N, bn);
  if (tiles == 0) return hipSuccess;
  const bool va = (K % 4 == 0) && aligned16(A), vb = (K % 4 == 0) && aligned16(B);
  const dim3 grid(tiles, 1);
  if (mask_src) BNS_GEMM_LAUNCH(true, true, 2, grid, M, N, K, A, K, B, K, C, N, K, va, vb, mask_src, alpha, m_dev, nullptr, Dropout{}, nullptr, 0, nullptr, 0);
  else BNS_GEMM_LAUNCH(true, true, 0, grid, M, N, K, A, K, B, K, C, N, K, va, vb, nullptr, alpha, m_dev, nullptr, Dropout{}, nullptr, 0, nullptr, 0);
  return hipGetLastError();
}

// ---- split-K -----------------------------------------------------------------------------------
// one round of resident workgroups: 256 compute units x 4 (LDS and registers allow four); measured
// against 512, 768, 1536 and 2048 on workloads 2 - 5
constexpr int kSplitTargetBlocks = 1024;
constexpr int kReduceGroup = 16;

static inline int splitk_chunk(int32_t M, int32_t N, int32_t K, int *splits_out) {
  const int tiles = (int)n_tiles(M, N, pick_bn(N));
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
splitk_reduce_kernel(const float *__restrict__ in, float *__restrict__ out, int64_t mn, int splits,
                     bool add_to_out) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= mn) return;
  const int z0 = blockIdx.y * kReduceGroup;
  const int z1 = min(splits, z0 + kReduceGroup);
  float sum = 0.f;
  for (int z = z0; z < z1; ++z) sum += in[(size_t)z * mn + i];
  if (add_to_out) sum += out[(size_t)blockIdx.y * mn + i];
  out[(size_t)blockIdx.y * mn + i] = sum;
}

hipError_t gemm_tn_splitk(int32_t M, int32_t N, int32_t K, const float *A, const float *B,
                          float *C, float *partials, bool accumulate, const int32_t *k_dev, hipStream_t s) {
  return gemm_tn_splitk_concat(M, N, K, A, nullptr, B, C, partials, accumulate, k_dev, s);
}

bool gemm_tn_concat_supported(int32_t M_half) { return M_half % BM == 0; }

// A2 != nullptr: C[2 M, N] = [A | A2]^T B with A, A2 [K, M] (M here is the width of one of them).
hipError_t gemm_tn_splitk_concat(int32_t M, int32_t N, int32_t K, const float *A, const float *A2, const float *B,
                                 float *C, float *partials, bool accumulate, const int32_t *k_dev,
                                 hipStream_t s) {
  const int M_half = M;
  if (A2) {
    if (!gemm_tn_concat_supported(M_half)) return hipErrorInvalidValue;
    M = 2 * M_half;
  }
  const int bn = pick_bn(N);
  const unsigned tiles = n_tiles(M, N, bn);
  if (tiles == 0) return hipSuccess;
  int splits;
  const int chunk = splitk_chunk(M, N, K, &splits);
  const bool va = (M_half % 4 == 0) && aligned16(A) && aligned16(A2), vb = (N % 4 == 0) && aligned16(B);
  const int64_t mn = (int64_t)M * N;
  float *dst = splits == 1 ? C : partials;
  const dim3 grid(tiles, splits);
  if (splits == 1 && accumulate)
    BNS_GEMM_LAUNCH(false, false, 3, grid, M, N, K, A, M_half, B, N, dst, N, chunk, va, vb, nullptr, 1.f, nullptr, k_dev, Dropout{}, A2, M_half, nullptr, 0);
  else
    BNS_GEMM_LAUNCH(false, false, 0, grid, M, N, K, A, M_half, B, N, dst, N, chunk, va, vb, nullptr, 1.f, nullptr, k_dev, Dropout{}, A2, M_half, nullptr, 0);
  // grouped, fixed-order reduction: partials -> level 2 -> ... -> C
  float *cur = partials;
  float *nxt = partials + (size_t)splits * mn;
  int n = splits;
  while (n > 1) {
    const int groups = (n + kReduceGroup - 1) / kReduceGroup;
    float *out = groups == 1 ? C : nxt;
    splitk_reduce_kernel<<<dim3((unsigned)((mn + 255) / 256), groups), 256, 0, s>>>(cur, out, mn, n,
                                                                                  accumulate && groups == 1);
    float *t = cur; cur = nxt; nxt = t;   // ping-pong (level >= 3 reuses the first buffer)
    n = groups;
  }
  return hipGetLastError();
}

}  // namespace bns
