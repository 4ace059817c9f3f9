// Loss summed over the inner nodes (Algorithm 1, loss step) with its gradient, the ReLU mask of
// the backward pass and the SGD update (Algorithm 1, update step).  The loss is reduced in a
// fixed order (per wavefront, per block, then one block over the block partials): two runs give
// the same bits.
#include <cmath>

#include "device_utils.hpp"
#include "kernels.hpp"

namespace bns {

constexpr int kT = 256;

__device__ __forceinline__ float block_sum_fixed(float x) {  // valid on thread 0
  __shared__ float part[kT / kWave];
  x = wave_sum(x);
  if (lane_id() == 0) part[threadIdx.x / kWave] = x;
  __syncthreads();
  float s = 0.f;
  if (threadIdx.x == 0)
#pragma unroll
    for (int w = 0; w < kT / kWave; ++w) s += part[w];
  __syncthreads();
  return s;
}

__global__ void __launch_bounds__(1024)
final_sum_kernel(const float *__restrict__ partials, int n, float *__restrict__ out) {
  __shared__ float part[1024 / kWave];
  float x = 0.f;
  for (int i = threadIdx.x; i < n; i += 1024) x += partials[i];
  x = wave_sum(x);
  if (lane_id() == 0) part[threadIdx.x / kWave] = x;
  __syncthreads();
  if (threadIdx.x == 0) {
    float s = 0.f;
    for (int w = 0; w < 1024 / kWave; ++w) s += part[w];
    *out = s;
  }
}

// softmax cross-entropy: one wavefront per node; loss_v = logsumexp(z_v) - z_v[y_v],
// dZ_v = softmax(z_v) - onehot(y_v).  Up to 256 classes a row lives in registers (one read).
__global__ void __launch_bounds__(kT)
softmax_ce_kernel(int n, int C, const float *__restrict__ logits, const int32_t *__restrict__ labels,
                  float *__restrict__ dZ, float *__restrict__ partials) {
  const int lane = lane_id();
  const int waves = gridDim.x * (kT / kWave);
  float loss_acc = 0.f;  // meaningful on lane 0
  const int v0 = blockIdx.x * (kT / kWave) + threadIdx.x / kWave;
  if (C <= 4 * kWave) {
    constexpr int R = 2;
    // two rows per step, their loads and reductions interleaved; the loss is still added row by
    // row in ascending order, so the sum does not depend on the pairing
    for (int v = v0; v < n; v += R * waves) {
      int row[R], y[R];
      float x[R][4], m[R], se[R];
#pragma unroll
      for (int r = 0; r < R; ++r) row[r] = v + r * waves;
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const bool ok = row[r] < n;
        y[r] = ok ? labels[row[r]] : -1;
        m[r] = -INFINITY;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int c = lane + k * kWave;
          x[r][k] = (ok && c < C) ? logits[(size_t)row[r] * C + c] : -INFINITY;
          m[r] = fmaxf(m[r], x[r][k]);
        }
      }
#pragma unroll
      for (int r = 0; r < R; ++r) m[r] = wave_max(m[r]);
      float zy[R];
#pragma unroll
      for (int r = 0; r < R; ++r) {
        se[r] = 0.f;
        zy[r] = 0.f;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int c = lane + k * kWave;
          if (c == y[r]) zy[r] = x[r][k];
          x[r][k] = c < C ? expf(x[r][k] - m[r]) : 0.f;
          se[r] += x[r][k];
        }
      }
#pragma unroll
      for (int r = 0; r < R; ++r) {
        se[r] = wave_sum(se[r]);
        zy[r] = wave_sum(zy[r]);  // exactly one lane holds z[y]; the others add zeros
      }
#pragma unroll
      for (int r = 0; r < R; ++r) {
        if (row[r] >= n) continue;
        float *g = dZ + (size_t)row[r] * C;
        const float inv = 1.f / se[r];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int c = lane + k * kWave;
          // a node outside the training set (negative label): no loss, zero gradient
          if (c < C) g[c] = y[r] < 0 ? 0.f : x[r][k] * inv - (c == y[r] ? 1.f : 0.f);
        }
        if (lane == 0 && y[r] >= 0) loss_acc += (m[r] + logf(se[r])) - zy[r];
      }
    }
  } else {
    for (int v = v0; v < n; v += waves) {
      const float *z = logits + (size_t)v * C;
      float *g = dZ + (size_t)v * C;
      const int y = labels[v];
      if (y < 0) {  // node outside the training set: no loss, zero gradient
        for (int c = lane; c < C; c += kWave) g[c] = 0.f;
        continue;
      }
      float m = -INFINITY;
      for (int c = lane; c < C; c += kWave) m = fmaxf(m, z[c]);
      m = wave_max(m);
      float se = 0.f;
      for (int c = lane; c < C; c += kWave) se += expf(z[c] - m);
      se = wave_sum(se);
      const float inv = 1.f / se;
      for (int c = lane; c < C; c += kWave) g[c] = expf(z[c] - m) * inv - (c == y ? 1.f : 0.f);
      if (lane == 0) loss_acc += (m + logf(se)) - z[y];
    }
  }
  const float s = block_sum_fixed(lane == 0 ? loss_acc : 0.f);
  if (threadIdx.x == 0) partials[blockIdx.x] = s;
}

// sigmoid binary cross-entropy over nodes x labels:
// loss = max(z,0) - z*y + log(1 + exp(-|z|)),  dZ = sigmoid(z) - y
__global__ void __launch_bounds__(kT)
sigmoid_bce_kernel(int64_t total, const float *__restrict__ logits, const uint8_t *__restrict__ labels,
                   float *__restrict__ dZ, float *__restrict__ partials) {
  const int64_t stride = (int64_t)gridDim.x * kT;
  float acc = 0.f;
  for (int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x; i < total; i += stride) {
    const float z = logits[i];
    if (labels[i] == 255) {  // entry outside the training set
      dZ[i] = 0.f;
      continue;
    }
    const float y = (float)labels[i];
    const float e = expf(-fabsf(z));
    acc += fmaxf(z, 0.f) - z * y + log1pf(e);
    const float sig = z >= 0.f ? 1.f / (1.f + e) : e / (1.f + e);
    dZ[i] = sig - y;
  }
  const float s = block_sum_fixed(acc);
  if (threadIdx.x == 0) partials[blockIdx.x] = s;
}

hipError_t loss_softmax_ce(int32_t n, int32_t C, const float *logits, const int32_t *labels,
                           float *dZ, float *partials, float *loss, hipStream_t s) {
  softmax_ce_kernel<<<kLossBlocks, kT, 0, s>>>(n, C, logits, labels, dZ, partials);
  final_sum_kernel<<<1, 1024, 0, s>>>(partials, kLossBlocks, loss);
  return hipGetLastError();
}

hipError_t loss_sigmoid_bce(int32_t n, int32_t C, const float *logits, const uint8_t *labels,
                            float *dZ, float *partials, float *loss, hipStream_t s) {
  sigmoid_bce_kernel<<<kLossBlocks, kT, 0, s>>>((int64_t)n * C, logits, labels, dZ, partials);
  final_sum_kernel<<<1, 1024, 0, s>>>(partials, kLossBlocks, loss);
  return hipGetLastError();
}

// one thread and one draw per element
__global__ void __launch_bounds__(kT)
dropout_inplace_kernel(int n_rows, int d, float *__restrict__ H, const Dropout drop) {
  const int64_t total = (int64_t)n_rows * d;
  const int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (i >= total) return;
  const int row = (int)(i / d), col = (int)(i - (int64_t)row * d);
  const float x = H[i];
  H[i] = dropout_keeps(drop, row, col) ? x * drop.scale : 0.f;
}

hipError_t dropout_inplace(int32_t n_rows, int32_t d, float *H, const Dropout &drop, hipStream_t s) {
  if (drop.scale == 0.f || n_rows <= 0) return hipSuccess;
  const int64_t total = (int64_t)n_rows * d;
  dropout_inplace_kernel<<<(unsigned)((total + kT - 1) / kT), kT, 0, s>>>(n_rows, d, H, drop);
  return hipGetLastError();
}

__global__ void __launch_bounds__(kT)
relu_mask_kernel(int64_t n, const float *__restrict__ dH, const float *__restrict__ H, float scale,
                 float *__restrict__ out) {
  const int64_t stride = (int64_t)gridDim.x * kT;
  for (int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x; i < n; i += stride)
    out[i] = H[i] > 0.f ? dH[i] * scale : 0.f;
}

hipError_t relu_mask(int64_t n, const float *dH, const float *H, float scale, float *out, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  int64_t blocks = (n + kT * 4 - 1) / (kT * 4);
  if (blocks > 65536) blocks = 65536;
  relu_mask_kernel<<<(unsigned)blocks, kT, 0, s>>>(n, dH, H, scale, out);
  return hipGetLastError();
}

__global__ void __launch_bounds__(kT)
sgd_kernel(int64_t n, float *__restrict__ W, const float *__restrict__ dW, float lr) {
  const int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (i < n) W[i] -= lr * dW[i];
}

// Adam (Kingma & Ba, 2015): m <- b1 m + (1-b1) g, v <- b2 v + (1-b2) g^2,
// w <- w - lr * (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps)
__global__ void __launch_bounds__(kT)
adam_kernel(int64_t n, float *__restrict__ W, const float *__restrict__ dW, float *__restrict__ m,
            float *__restrict__ v, float lr, float b1, float b2, float eps, float c1, float c2) {
  const int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (i >= n) return;
  const float g = dW[i];
  const float mi = b1 * m[i] + (1.f - b1) * g;
  const float vi = b2 * v[i] + (1.f - b2) * g * g;
  m[i] = mi;
  v[i] = vi;
  W[i] -= lr * (mi * c1) / (sqrtf(vi * c2) + eps);
}

hipError_t adam_update(int64_t n, float *W, const float *dW, float *m, float *v, float lr, float b1,
                       float b2, float eps, int32_t t, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  const float c1 = (float)(1.0 / (1.0 - pow((double)b1, (double)t)));
  const float c2 = (float)(1.0 / (1.0 - pow((double)b2, (double)t)));
  adam_kernel<<<(unsigned)((n + kT - 1) / kT), kT, 0, s>>>(n, W, dW, m, v, lr, b1, b2, eps, c1, c2);
  return hipGetLastError();
}

__global__ void counter_kernel(uint32_t *counter, uint32_t value, bool bump) {
  *counter = bump ? *counter + 1u : value;
}
hipError_t set_counter(uint32_t *counter, uint32_t value, hipStream_t s) {
  counter_kernel<<<1, 1, 0, s>>>(counter, value, false);
  return hipGetLastError();
}
hipError_t bump_counter(uint32_t *counter, hipStream_t s) {
  counter_kernel<<<1, 1, 0, s>>>(counter, 0u, true);
  return hipGetLastError();
}

hipError_t sgd_update(int64_t n, float *W, const float *dW, float lr, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  sgd_kernel<<<(unsigned)((n + kT - 1) / kT), kT, 0, s>>>(n, W, dW, lr);
  return hipGetLastError();
}

}  // namespace bns
