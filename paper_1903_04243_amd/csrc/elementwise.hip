// Small row-wise kernels: the loss head, the seed rows of the Jacobians, and a transpose.
// Each row is handled by one 64-lane wave; lanes stride over the d_L classes and combine with
// wave reductions (Section 3.4: a reduction inside the loop body keeps reducing over its own
// axis after vectorisation; it never reduces over the iteration index).
#include "common.h"

namespace pfg {

namespace {

constexpr int kThreads = 256;
constexpr int kWavesPerBlock = kThreads / 64;

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// Max and log-sum-exp denominator of one row of logits, by the whole wave.
__device__ __forceinline__ void row_softmax_stats(const float *y, int n, int lane, float &mx,
                                                  float &den) {
  float m = -INFINITY;
  for (int j = lane; j < n; j += 64) m = fmaxf(m, y[j]);
  mx = wave_max(m);
  float s = 0.f;
  for (int j = lane; j < n; j += 64) s += expf(y[j] - mx);
  den = wave_sum(s);
}

__global__ __launch_bounds__(kThreads) void head_softmax_ce_kernel(const float *y,
                                                                   const int32_t *labels,
                                                                   int64_t B, int n, float *delta,
                                                                   float *loss) {
  const int lane = threadIdx.x & 63;
  const int64_t b = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
  if (b >= B) return;
  const float *row = y + b * n;
  float mx, den;
  row_softmax_stats(row, n, lane, mx, den);
  const int label = labels[b];
  const float inv = 1.f / den;
  // delta[label] = p[label] - 1 = -(sum of the other classes' terms) / den, which avoids the
  // cancellation when p[label] is close to one
  float others = 0.f;
  for (int j = lane; j < n; j += 64)
    if (j != label) others += expf(row[j] - mx);
  others = wave_sum(others);
  for (int j = lane; j < n; j += 64) {
    const float p = expf(row[j] - mx) * inv;
    delta[b * n + j] = (j == label) ? -others * inv : p;
  }
  if (loss && lane == 0) {
    // -log p[label] = log(den) - (y[label] - max); an out-of-range label reads nothing
    const float yl = (label >= 0 && label < n) ? row[label] : mx;
    loss[b] = logf(den) - (yl - mx);
  }
}

// G[b, s, :] = r                      (head = logits)
//            = p * (r - <r, p>)       (head = softmax; this is sum_c r[c] * p[c] (e_c - p))
// with r = seed row (b, s), or e_s when seeds == nullptr, and p = softmax(y[b, :]).
__global__ __launch_bounds__(kThreads) void seed_rows_kernel(const float *y, const float *seeds,
                                                             int64_t seed_batch_stride, int64_t B,
                                                             int64_t S, int n, int head, float *G) {
  const int lane = threadIdx.x & 63;
  const int64_t row_id = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
  if (row_id >= B * S) return;
  const int64_t b = row_id / S, s = row_id % S;
  const float *r = seeds ? seeds + b * seed_batch_stride + s * n : nullptr;
  float *out = G + row_id * n;
  if (head == 0) {
    for (int j = lane; j < n; j += 64) out[j] = r ? r[j] : (j == s ? 1.f : 0.f);
    return;
  }
  const float *yrow = y + b * n;
  float mx, den;
  row_softmax_stats(yrow, n, lane, mx, den);
  const float inv = 1.f / den;
  float dot = 0.f;
  for (int j = lane; j < n; j += 64) {
    const float rj = r ? r[j] : (j == s ? 1.f : 0.f);
    dot += rj * expf(yrow[j] - mx) * inv;
  }
  dot = wave_sum(dot);
  for (int j = lane; j < n; j += 64) {
    const float rj = r ? r[j] : (j == s ? 1.f : 0.f);
    out[j] = expf(yrow[j] - mx) * inv * (rj - dot);
  }
}

// dst[c, r] = src[r, c] through a padded 32 x 32 LDS tile.
__global__ __launch_bounds__(kThreads) void transpose_kernel(const void *src, int src_bf16, int R,
                                                             int C, float *dst) {
  __shared__ float tile[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
  const int tiles_c = (C + 31) / 32;
  const int c0 = (blockIdx.x % tiles_c) * 32, r0 = (blockIdx.x / tiles_c) * 32;
  for (int k = ty; k < 32; k += 8) {
    const int r = r0 + k, c = c0 + tx;
    float v = 0.f;
    if (r < R && c < C) {
      const int64_t idx = (int64_t)r * C + c;
      v = src_bf16 ? (float)static_cast<const __bf16 *>(src)[idx]
                   : static_cast<const float *>(src)[idx];
    }
    tile[k][tx] = v;
  }
  __syncthreads();
  for (int k = ty; k < 32; k += 8) {
    const int c = c0 + k, r = r0 + tx;
    if (r < R && c < C) dst[(int64_t)c * R + r] = tile[tx][k];
  }
}

}  // namespace

hipError_t launch_head_softmax_ce(const float *y, const int32_t *labels, int64_t B, int32_t n,
                                  float *delta, float *loss, hipStream_t stream) {
  if (B <= 0) return hipSuccess;
  const int64_t blocks = (B + kWavesPerBlock - 1) / kWavesPerBlock;
  PFG_KERNEL(head_softmax_ce_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, y,
                     labels, B, n, delta, loss);
  return hipGetLastError();
}

hipError_t launch_seed_rows(const float *y, const float *seeds, int64_t seed_batch_stride,
                            int64_t B, int64_t S, int32_t n, int32_t head, float *G,
                            hipStream_t stream) {
  if (B * S <= 0) return hipSuccess;
  const int64_t blocks = (B * S + kWavesPerBlock - 1) / kWavesPerBlock;
  PFG_KERNEL(seed_rows_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, y, seeds,
                     seed_batch_stride, B, S, n, head, G);
  return hipGetLastError();
}

hipError_t launch_transpose(const void *src, int32_t src_bf16, int32_t R, int32_t C, float *dst,
                            hipStream_t stream) {
  if (R <= 0 || C <= 0) return hipSuccess;
  const int64_t blocks = (int64_t)((R + 31) / 32) * ((C + 31) / 32);
  PFG_KERNEL(transpose_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, src,
                     src_bf16, R, C, dst);
  return hipGetLastError();
}

}  // namespace pfg
