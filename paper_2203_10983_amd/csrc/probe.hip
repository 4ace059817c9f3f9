// Instrumentation: the bare access pattern of the aggregate, without its arithmetic.  Every wavefront
// sums `per_wave` rows of a table picked by an index list (no weights, no row structure, one row stored
// per wavefront), with the same 16-byte loads and the same number of loads in flight as the aggregate
// kernels.  Timed beside a training step it gives this machine's ceiling for gathering that many rows
// of that width from a table of that size, which is what bounds Eq. 1 on a graph without locality.
#include <hip/hip_runtime.h>

#include "../../include/bns_gcn.h"
#include "device_utils.hpp"

namespace bns {

typedef float v4f __attribute__((ext_vector_type(4)));

template <int LPR>
__global__ void __launch_bounds__(256)
probe_gather_kernel(const float *__restrict__ table, int32_t d, const int32_t *__restrict__ idx, int64_t n_idx,
                    int32_t per_wave, float *__restrict__ out) {
  constexpr int EP = kWave / LPR, UNR = 8;  // rows per load instruction, load instructions in flight
  const int lane = lane_id();
  const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int64_t b0 = wave * per_wave;
  const int64_t b1 = b0 + per_wave < n_idx ? b0 + per_wave : n_idx;
  const int g = lane / LPR, sl = lane % LPR;
  v4f acc = {0.f, 0.f, 0.f, 0.f};
  for (int64_t base = b0; base < b1; base += kWave) {
    const int cnt = (int)(b1 - base < kWave ? b1 - base : kWave);
    const int c = lane < cnt ? idx[base + lane] : 0;
    for (int j = 0; j < cnt; j += UNR * EP) {
      v4f v[UNR];
#pragma unroll
      for (int t = 0; t < UNR; ++t) {
        const int jj = j + t * EP + g;
        const int cc = __shfl(c, jj & (kWave - 1), kWave);
        v[t] = jj < cnt ? reinterpret_cast<const v4f *>(table + (size_t)cc * d)[sl] : v4f{0.f, 0.f, 0.f, 0.f};
      }
#pragma unroll
      for (int t = 0; t < UNR; ++t) acc += v[t];
    }
  }
  // the lane groups hold partial sums of the same row slice: fold them, store one d-float row
#pragma unroll
  for (int off = LPR; off < kWave; off <<= 1) {
    acc.x += __shfl_xor(acc.x, off, kWave);
    acc.y += __shfl_xor(acc.y, off, kWave);
    acc.z += __shfl_xor(acc.z, off, kWave);
    acc.w += __shfl_xor(acc.w, off, kWave);
  }
  if (b0 < n_idx && g == 0) reinterpret_cast<v4f *>(out + wave * d)[sl] = acc;
}

// The fp32 matrix instruction of the update (Eq. 2) with nothing else in the loop: every wavefront
// issues iters x 8 x NACC v_mfma_f32_32x32x2_f32 on NACC independent accumulators.  How many of them a
// SIMD issues per second depends on the wavefronts resident per SIMD and on NACC; the GEMM tiles
// are shaped after what this measures.
typedef float floatx16 __attribute__((ext_vector_type(16)));

template <int NACC>
__global__ void __launch_bounds__(1024) probe_mfma_kernel(float *__restrict__ out, int iters, float a0, float b0) {
  floatx16 acc[NACC];
#pragma unroll
  for (int i = 0; i < NACC; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  const float a = a0 + threadIdx.x * 1e-6f, b = b0;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
      for (int i = 0; i < NACC; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NACC; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  // one float per workgroup, so that the products are not optimised away
  if (threadIdx.x == 0) out[blockIdx.x] = s;
}

}  // namespace bns

extern "C" bns_status bns_probe_mfma(int32_t n_acc, int32_t waves_per_block, int32_t blocks, int32_t iters,
                                     float *out, void *stream) {
  using namespace bns;
  if (!out || blocks < 1 || iters < 0 || waves_per_block < 1 || waves_per_block > 16) return BNS_EINVAL;
  if (n_acc != 1 && n_acc != 2 && n_acc != 3 && n_acc != 4 && n_acc != 6) return BNS_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const unsigned threads = (unsigned)waves_per_block * kWave;
  switch (n_acc) {
    case 1: probe_mfma_kernel<1><<<(unsigned)blocks, threads, 0, s>>>(out, iters, 1.0f, 0.5f); break;
    case 2: probe_mfma_kernel<2><<<(unsigned)blocks, threads, 0, s>>>(out, iters, 1.0f, 0.5f); break;
    case 3: probe_mfma_kernel<3><<<(unsigned)blocks, threads, 0, s>>>(out, iters, 1.0f, 0.5f); break;
    case 4: probe_mfma_kernel<4><<<(unsigned)blocks, threads, 0, s>>>(out, iters, 1.0f, 0.5f); break;
    default: probe_mfma_kernel<6><<<(unsigned)blocks, threads, 0, s>>>(out, iters, 1.0f, 0.5f); break;
  }
  if (hipGetLastError() != hipSuccess) {
    (void)hipGetLastError();
    return BNS_EHIP;
  }
  return BNS_OK;
}

extern "C" bns_status bns_probe_gather(const float *table, int64_t n_rows, int32_t d, const int32_t *idx,
                                       int64_t n_idx, int32_t per_wave, float *out, void *stream) {
  using namespace bns;
  if (!table || !idx || !out || n_rows < 1 || n_idx < 0 || per_wave < 1) return BNS_EINVAL;
  if (d != 16 && d != 32 && d != 64 && d != 128 && d != 256) return BNS_EINVAL;
  if (n_idx == 0) return BNS_OK;
  const int64_t waves = (n_idx + per_wave - 1) / per_wave;
  const int64_t blocks = (waves + 3) / 4;
  if (blocks > 0x7fffffffLL) return BNS_EOVERFLOW;
  hipStream_t s = static_cast<hipStream_t>(stream);
  switch (d) {
    case 16: probe_gather_kernel<4><<<(unsigned)blocks, 256, 0, s>>>(table, d, idx, n_idx, per_wave, out); break;
    case 32: probe_gather_kernel<8><<<(unsigned)blocks, 256, 0, s>>>(table, d, idx, n_idx, per_wave, out); break;
    case 64: probe_gather_kernel<16><<<(unsigned)blocks, 256, 0, s>>>(table, d, idx, n_idx, per_wave, out); break;
    case 128: probe_gather_kernel<32><<<(unsigned)blocks, 256, 0, s>>>(table, d, idx, n_idx, per_wave, out); break;
    default: probe_gather_kernel<64><<<(unsigned)blocks, 256, 0, s>>>(table, d, idx, n_idx, per_wave, out); break;
  }
  if (hipGetLastError() != hipSuccess) {
    (void)hipGetLastError();
    return BNS_EHIP;
  }
  return BNS_OK;
}
