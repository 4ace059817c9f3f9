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

}  // namespace bns

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
