// Kernels of the convolutional blocks that are not matrix products.  Images are [B, h, w, c] with
// the channel index fastest.  A "same"-size k x k convolution becomes a product once every output
// position has its k * k * c input patch laid out as a row (Section 3.4's convolution rule folds the
// example index into the batch of positions: rows (b, y, x)); the per-example filter gradient is a
// product per example over the positions, for which the patches are also kept with the position
// index fastest.
#include <algorithm>

#include "common.h"

namespace pfg {

namespace {

constexpr int kThreads = 256;

inline unsigned capped_blocks(int64_t work_items) {
  const int64_t blocks = (work_items + kThreads - 1) / kThreads;
  return (unsigned)(blocks < (1 << 20) ? blocks : (1 << 20));
}

// P[(b, y, x), (ky, kx, c)] = in[b, y + ky - p, x + kx - p, c] (zero outside the image).
// ROWS_ARE_POSITIONS: P is [B h w, k k c] (a workgroup row walks a patch); otherwise the transposed
// per-example layout [B, k k c, h w] (a workgroup row walks the positions).  The second grid index
// is the example, the first a chunk of kRows rows of that example's matrix; the threads of one row
// slot take consecutive entries, so the divisions that locate a row are done once per slot and the
// rest is 32-bit arithmetic.
constexpr int kRows = 4;      // row slots per workgroup (64 threads each)

template <bool ROWS_ARE_POSITIONS>
__global__ __launch_bounds__(kThreads) void im2col_kernel(const float *in, int h, int w, int c, int k,
                                                          float *out) {
  const int p = (k - 1) / 2, hw = h * w, kkc = k * k * c;
  const int nrows = ROWS_ARE_POSITIONS ? hw : kkc, ncols = ROWS_ARE_POSITIONS ? kkc : hw;
  const int64_t b = blockIdx.y;
  const int row = blockIdx.x * kRows + (threadIdx.x >> 6);
  if (row >= nrows) return;
  const float *img = in + b * (int64_t)hw * c;
  float *orow = out + (b * nrows + row) * (int64_t)ncols;
  const bool aligned = ((reinterpret_cast<uintptr_t>(in) | reinterpret_cast<uintptr_t>(out)) & 15) == 0;
  if (ROWS_ARE_POSITIONS && c % 4 == 0 && aligned) {
    // four channels at a time: a 16-byte piece never straddles two filter taps
    const int y = row / w, x = row - y * w;
    for (int e = (threadIdx.x & 63) * 4; e < ncols; e += 256) {
      const int kyx = e / c, ch = e - kyx * c;
      const int ky = kyx / k, kx = kyx - ky * k;
      const int yy = y + ky - p, xx = x + kx - p;
      f32x4 v = {0.f, 0.f, 0.f, 0.f};
      if (yy >= 0 && yy < h && xx >= 0 && xx < w)
        v = *reinterpret_cast<const f32x4 *>(img + (yy * w + xx) * c + ch);
      *reinterpret_cast<f32x4 *>(orow + e) = v;
    }
  } else if (!ROWS_ARE_POSITIONS && hw % 4 == 0 && aligned) {
    // four positions at a time: strided reads, one 16-byte store
    const int kyx = row / c, ch = row - kyx * c;
    const int ky = kyx / k, kx = kyx - ky * k;
    for (int pos = (threadIdx.x & 63) * 4; pos < ncols; pos += 256) {
      f32x4 v;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int y = (pos + q) / w, x = (pos + q) - y * w;
        const int yy = y + ky - p, xx = x + kx - p;
        v[q] = (yy >= 0 && yy < h && xx >= 0 && xx < w) ? img[(yy * w + xx) * c + ch] : 0.f;
      }
      *reinterpret_cast<f32x4 *>(orow + pos) = v;
    }
  } else if (ROWS_ARE_POSITIONS) {
    const int y = row / w, x = row - y * w;
    for (int e = threadIdx.x & 63; e < ncols; e += 64) {
      const int kyx = e / c, ch = e - kyx * c;
      const int ky = kyx / k, kx = kyx - ky * k;
      const int yy = y + ky - p, xx = x + kx - p;
      orow[e] = (yy >= 0 && yy < h && xx >= 0 && xx < w) ? img[(yy * w + xx) * c + ch] : 0.f;
    }
  } else {
    const int kyx = row / c, ch = row - kyx * c;
    const int ky = kyx / k, kx = kyx - ky * k;
    for (int pos = threadIdx.x & 63; pos < ncols; pos += 64) {
      const int y = pos / w, x = pos - y * w;
      const int yy = y + ky - p, xx = x + kx - p;
      orow[pos] = (yy >= 0 && yy < h && xx >= 0 && xx < w) ? img[(yy * w + xx) * c + ch] : 0.f;
    }
  }
}

// P [B h w, k k c] as one flat array when a patch row is not a whole number of 16-byte pieces (a
// single-channel image: rows of k k values): consecutive threads take consecutive groups of four
// values, whichever rows they fall in, so the stores stay 16 bytes wide and contiguous.
__global__ __launch_bounds__(kThreads) void im2col_flat_kernel(const float *in, int64_t B, int h, int w, int c,
                                                               int k, float *out) {
  const int p = (k - 1) / 2, hw = h * w, kkc = k * k * c;
  const int64_t total = B * hw * (int64_t)kkc;
  const int64_t step = (int64_t)gridDim.x * kThreads * 4;
  for (int64_t e0 = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * 4; e0 < total; e0 += step) {
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int64_t e = e0 + q;
      if (e >= total) break;
      const int64_t row = e / kkc;
      const int t = (int)(e - row * kkc);
      const int kyx = t / c, ch = t - kyx * c;
      const int ky = kyx / k, kx = kyx - ky * k;
      const int64_t b = row / hw;
      const int pos = (int)(row - b * hw);
      const int y = pos / w, x = pos - y * w;
      const int yy = y + ky - p, xx = x + kx - p;
      if (yy >= 0 && yy < h && xx >= 0 && xx < w) v[q] = in[(b * hw + yy * w + xx) * c + ch];
    }
    if (e0 + 4 <= total) {
      *reinterpret_cast<f32x4 *>(out + e0) = v;
    } else {
      for (int q = 0; e0 + q < total; ++q) out[e0 + q] = v[q];
    }
  }
}

// Both layouts of a small image's patches in one launch, through LDS: a workgroup copies the whole
// image of its example into LDS (h w c <= kLdsImage floats) and writes one slab of P[b] and of PT[b]
// as flat runs of 16-byte stores, finding the source of each value by counting (tap, channel,
// position) up from the slab's first entry instead of dividing per value.  For images whose patch
// rows are not whole 16-byte pieces (a single channel), where the other kernels gather value by
// value from global memory.  P[b] and PT[b] must be 16-byte aligned (h w k k c a multiple of 4).
constexpr int kLdsImage = 8192;

// n / d for 0 <= n < 2^24 and d >= 1 with the reciprocal given: the float product is off by one at
// most, which the remainder shows (a 32-bit division by a run-time divisor costs ten times as much,
// and the kernel below is made of them)
__device__ __forceinline__ int div_small(int n, int d, float inv) {
  int q = (int)((float)n * inv);
  const int r = n - q * d;
  if (r < 0) --q;
  if (r >= d) ++q;
  return q;
}

__global__ __launch_bounds__(kThreads) void im2col_lds_kernel(const float *in, int h, int w, int c, int k,
                                                              float *P, float *PT) {
  __shared__ float img[kLdsImage];
  const int p = (k - 1) / 2, hw = h * w, kkc = k * k * c, n = hw * c;
  const float inv_kkc = 1.f / (float)kkc, inv_hw = 1.f / (float)hw, inv_w = 1.f / (float)w, inv_c = 1.f / (float)c,
              inv_k = 1.f / (float)k;
  const int64_t b = blockIdx.y;
  const float *src = in + b * n;
  for (int i = threadIdx.x; i < n; i += kThreads) img[i] = src[i];
  __syncthreads();
  const int total = hw * kkc;                       // values of P[b] (and of PT[b])
  const int per = ((total / 4 + gridDim.x - 1) / gridDim.x) * 4;
  const int e_begin = blockIdx.x * per, e_end = min(total, e_begin + per);
  if (P) {
    float *out = P + b * total;
    for (int e0 = e_begin + 4 * threadIdx.x; e0 < e_end; e0 += 4 * kThreads) {
      // entry e0 of [h w, k k c]: position, tap and channel; then counted up
      int pos = div_small(e0, kkc, inv_kkc), t = e0 - pos * kkc;
      int y = div_small(pos, w, inv_w), x = pos - y * w;
      int kyx = div_small(t, c, inv_c), ch = t - kyx * c;
      int ky = div_small(kyx, k, inv_k), kx = kyx - ky * k;
      f32x4 v;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int yy = y + ky - p, xx = x + kx - p;
        v[q] = (yy >= 0 && yy < h && xx >= 0 && xx < w) ? img[(yy * w + xx) * c + ch] : 0.f;
        if (++ch == c) {
          ch = 0;
          if (++kx == k) {
            kx = 0;
            if (++ky == k) {
              ky = 0;
              if (++x == w) { x = 0; ++y; }
            }
          }
        }
      }
      *reinterpret_cast<f32x4 *>(out + e0) = v;
    }
  }
  if (PT) {
    float *out = PT + b * total;
    for (int e0 = e_begin + 4 * threadIdx.x; e0 < e_end; e0 += 4 * kThreads) {
      // entry e0 of [k k c, h w]
      int t = div_small(e0, hw, inv_hw), pos = e0 - t * hw;
      int y = div_small(pos, w, inv_w), x = pos - y * w;
      int kyx = div_small(t, c, inv_c), ch = t - kyx * c;
      int ky = div_small(kyx, k, inv_k), kx = kyx - ky * k;
      f32x4 v;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int yy = y + ky - p, xx = x + kx - p;
        v[q] = (yy >= 0 && yy < h && xx >= 0 && xx < w) ? img[(yy * w + xx) * c + ch] : 0.f;
        if (++x == w) {
          x = 0;
          if (++y == h) {
            y = 0;
            if (++ch == c) {
              ch = 0;
              if (++kx == k) { kx = 0; ++ky; }
            }
          }
        }
      }
      *reinterpret_cast<f32x4 *>(out + e0) = v;
    }
  }
}

// The position-fastest layout PT [B, k k c, h w] for images with several channels.  Reading the image
// position by position for one channel touches one value per 4 c bytes; instead a workgroup takes
// one filter tap of one example and a run of kPosRun positions, reads their c channels (contiguous
// in the image) into LDS and writes them out transposed, c rows of kPosRun consecutive positions.
constexpr int kPosRun = 64;
constexpr int kMaxTiledC = 128;      // LDS: kPosRun x (c + 1) floats

__global__ __launch_bounds__(kThreads) void im2col_pt_tiled_kernel(const float *in, int h, int w, int c, int k,
                                                                   float *out) {
  __shared__ float tile[kPosRun * (kMaxTiledC + 1)];
  const int p = (k - 1) / 2, hw = h * w, kkc = k * k * c;
  const int tap = blockIdx.x, pos0 = blockIdx.y * kPosRun;
  const int64_t b = blockIdx.z;
  const int ky = tap / k, kx = tap - ky * k;
  const int npos = min(kPosRun, hw - pos0);
  const float *img = in + b * (int64_t)hw * c;
  const int ts = c + 1;
  const bool vec = c % 4 == 0 && hw % 4 == 0 &&
                   ((reinterpret_cast<uintptr_t>(in) | reinterpret_cast<uintptr_t>(out)) & 15) == 0;
  if (vec) {
    // 16 bytes of channels per load, 16 bytes of positions per store
    const int c4 = c / 4;
    for (int idx = threadIdx.x; idx < npos * c4; idx += kThreads) {
      const int pl = idx / c4, ch = (idx - pl * c4) * 4;
      const int pos = pos0 + pl;
      const int y = pos / w, x = pos - y * w;
      const int yy = y + ky - p, xx = x + kx - p;
      f32x4 v = {0.f, 0.f, 0.f, 0.f};
      if (yy >= 0 && yy < h && xx >= 0 && xx < w) v = *reinterpret_cast<const f32x4 *>(img + (yy * w + xx) * c + ch);
#pragma unroll
      for (int q = 0; q < 4; ++q) tile[pl * ts + ch + q] = v[q];
    }
    __syncthreads();
    float *obase = out + (b * kkc + (int64_t)tap * c) * hw + pos0;
    for (int idx = threadIdx.x; idx < c * (kPosRun / 4); idx += kThreads) {
      const int ch = idx / (kPosRun / 4), pl = (idx - ch * (kPosRun / 4)) * 4;
      if (pl >= npos) continue;                    // npos is a multiple of 4 here
      f32x4 v;
#pragma unroll
      for (int q = 0; q < 4; ++q) v[q] = tile[(pl + q) * ts + ch];
      *reinterpret_cast<f32x4 *>(obase + (int64_t)ch * hw + pl) = v;
    }
    return;
  }
  for (int idx = threadIdx.x; idx < npos * c; idx += kThreads) {
    const int pl = idx / c, ch = idx - pl * c;
    const int pos = pos0 + pl;
    const int y = pos / w, x = pos - y * w;
    const int yy = y + ky - p, xx = x + kx - p;
    tile[pl * ts + ch] = (yy >= 0 && yy < h && xx >= 0 && xx < w) ? img[(yy * w + xx) * c + ch] : 0.f;
  }
  __syncthreads();
  float *obase = out + (b * kkc + (int64_t)tap * c) * hw + pos0;
  for (int idx = threadIdx.x; idx < c * kPosRun; idx += kThreads) {
    const int ch = idx / kPosRun, pl = idx - ch * kPosRun;
    if (pl < npos) obase[(int64_t)ch * hw + pl] = tile[pl * ts + ch];
  }
}

// a = relu(z); pooled = max of each 2 x 2 window, which = position of the first maximum in the
// order (0,0), (0,1), (1,0), (1,1).  One thread per pooled cell, channel fastest.
__global__ __launch_bounds__(kThreads) void relu_pool_kernel(const float *z, int64_t B, int h, int w, int c,
                                                             float *pooled, uint8_t *which) {
  const int ho = h / 2, wo = w / 2;
  const int64_t total = B * ho * wo * c;
  const int64_t step = (int64_t)gridDim.x * kThreads;
  if (c % 4 == 0 && ((reinterpret_cast<uintptr_t>(z) | reinterpret_cast<uintptr_t>(pooled)) & 15) == 0 &&
      (reinterpret_cast<uintptr_t>(which) & 3) == 0) {
    // four channels per thread: 16-byte loads and stores, the four window indices as one word
    const int c4 = c / 4;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total / 4; i += step) {
      const int ch = (int)(i % c4) * 4;
      int64_t r = i / c4;
      const int xo = (int)(r % wo);
      r /= wo;
      const int yo = (int)(r % ho);
      const int64_t b = r / ho;
      f32x4 best = {-1.f, -1.f, -1.f, -1.f};
      uint32_t arg = 0;
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        const f32x4 v = *reinterpret_cast<const f32x4 *>(
            z + ((b * h + 2 * yo + (d >> 1)) * w + 2 * xo + (d & 1)) * c + ch);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const float a = v[q] > 0.f ? v[q] : 0.f;
          if (a > best[q]) {
            best[q] = a;
            arg = (arg & ~(0xffu << (8 * q))) | ((uint32_t)d << (8 * q));
          }
        }
      }
      *reinterpret_cast<f32x4 *>(pooled + 4 * i) = best;
      *reinterpret_cast<uint32_t *>(which + 4 * i) = arg;
    }
    return;
  }
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += step) {
    const int ch = (int)(i % c);
    int64_t r = i / c;
    const int xo = (int)(r % wo);
    r /= wo;
    const int yo = (int)(r % ho);
    const int64_t b = r / ho;
    float best = -1.f;
    int arg = 0;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      const float v = z[((b * h + 2 * yo + (d >> 1)) * w + 2 * xo + (d & 1)) * c + ch];
      const float a = v > 0.f ? v : 0.f;
      if (a > best) { best = a; arg = d; }
    }
    pooled[i] = best;
    which[i] = (uint8_t)arg;
  }
}

// Cotangent of the conv pre-activations from the cotangent of the pooled output: the window entry
// that gave the maximum receives it if it was positive (relu'), the others receive zero.  Every
// entry of dz is written.
__global__ __launch_bounds__(kThreads) void unpool_mask_kernel(const float *dpooled, const float *pooled,
                                                               const uint8_t *which, int64_t B, int h,
                                                               int w, int c, float *dz) {
  const int ho = h / 2, wo = w / 2;
  const int64_t total = B * ho * wo * c;
  const int64_t step = (int64_t)gridDim.x * kThreads;
  if (c % 4 == 0 && (reinterpret_cast<uintptr_t>(which) & 3) == 0 &&
      ((reinterpret_cast<uintptr_t>(dpooled) | reinterpret_cast<uintptr_t>(pooled) |
        reinterpret_cast<uintptr_t>(dz)) & 15) == 0) {
    const int c4 = c / 4;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total / 4; i += step) {
      const int ch = (int)(i % c4) * 4;
      int64_t r = i / c4;
      const int xo = (int)(r % wo);
      r /= wo;
      const int yo = (int)(r % ho);
      const int64_t b = r / ho;
      const f32x4 p = *reinterpret_cast<const f32x4 *>(pooled + 4 * i);
      const f32x4 dp = *reinterpret_cast<const f32x4 *>(dpooled + 4 * i);
      const uint32_t arg = *reinterpret_cast<const uint32_t *>(which + 4 * i);
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        f32x4 out;
#pragma unroll
        for (int q = 0; q < 4; ++q)
          out[q] = (((arg >> (8 * q)) & 0xffu) == (uint32_t)d && p[q] > 0.f) ? dp[q] : 0.f;
        *reinterpret_cast<f32x4 *>(dz + ((b * h + 2 * yo + (d >> 1)) * w + 2 * xo + (d & 1)) * c + ch) = out;
      }
    }
    return;
  }
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += step) {
    const int ch = (int)(i % c);
    int64_t r = i / c;
    const int xo = (int)(r % wo);
    r /= wo;
    const int yo = (int)(r % ho);
    const int64_t b = r / ho;
    const float g = pooled[i] > 0.f ? dpooled[i] : 0.f;
    const int arg = which[i];
#pragma unroll
    for (int d = 0; d < 4; ++d)
      dz[((b * h + 2 * yo + (d >> 1)) * w + 2 * xo + (d & 1)) * c + ch] = (d == arg) ? g : 0.f;
  }
}

// The same with the bias gradient db[b, ch] = sum over the positions of dz[b, ., ., ch] produced on
// the way.  A window hands its cotangent to at most one of its entries, so the sum runs over the
// pooled cells.  One workgroup per example; a thread stays with one group of four channels (the
// threads in use are a multiple of the number of groups), and the threads of a group are added in a
// fixed order through LDS, so the result does not depend on timing.  c % 4 == 0, c <= 4 kThreads,
// 16-byte aligned operands.
__global__ __launch_bounds__(kThreads) void unpool_mask_sum_kernel(const float *dpooled, const float *pooled,
                                                                   const uint8_t *which, int h, int w, int c,
                                                                   float *dz, float *db) {
  __shared__ f32x4 part[kThreads];
  const int64_t b = blockIdx.x;
  const int ho = h / 2, wo = w / 2, c4 = c / 4;
  const int units = ho * wo * c4;
  const int lanes = (kThreads / c4) * c4;
  const int tid = threadIdx.x;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  if (tid < lanes) {
    const int ch = (tid % c4) * 4;
    for (int u = tid; u < units; u += lanes) {
      const int cell = u / c4;
      const int xo = cell % wo, yo = cell / wo;
      const int64_t i = b * units + u;
      const f32x4 p = *reinterpret_cast<const f32x4 *>(pooled + 4 * i);
      const f32x4 dp = *reinterpret_cast<const f32x4 *>(dpooled + 4 * i);
      const uint32_t arg = *reinterpret_cast<const uint32_t *>(which + 4 * i);
      f32x4 live;
#pragma unroll
      for (int q = 0; q < 4; ++q) live[q] = p[q] > 0.f ? dp[q] : 0.f;
      acc += live;
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        f32x4 out;
#pragma unroll
        for (int q = 0; q < 4; ++q) out[q] = (((arg >> (8 * q)) & 0xffu) == (uint32_t)d) ? live[q] : 0.f;
        *reinterpret_cast<f32x4 *>(dz + ((b * h + 2 * yo + (d >> 1)) * w + 2 * xo + (d & 1)) * c + ch) = out;
      }
    }
  }
  part[tid] = acc;
  __syncthreads();
  if (tid < c4) {
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    for (int t = tid; t < lanes; t += c4) s += part[t];
    *reinterpret_cast<f32x4 *>(db + b * c + 4 * tid) = s;
  }
}

// din[b, yy, xx, ch] = sum over the patches that contain the pixel of their cotangent entry:
// dP[(b, yy - ky + p, xx - kx + p), (ky, kx, ch)].  A gather in a fixed order (no atomics).
__global__ __launch_bounds__(kThreads) void col2im_kernel(const float *dP, int64_t B, int h, int w, int c,
                                                          int k, float *din) {
  const int p = (k - 1) / 2, kkc = k * k * c;
  const int64_t total = B * h * w * c;
  const int64_t step = (int64_t)gridDim.x * kThreads;
  if (c % 4 == 0 && ((reinterpret_cast<uintptr_t>(dP) | reinterpret_cast<uintptr_t>(din)) & 15) == 0) {
    // four channels per thread, the same taps in the same order
    const int c4 = c / 4;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total / 4; i += step) {
      const int ch = (int)(i % c4) * 4;
      int64_t r = i / c4;
      const int xx = (int)(r % w);
      r /= w;
      const int yy = (int)(r % h);
      const int64_t b = r / h;
      f32x4 s = {0.f, 0.f, 0.f, 0.f};
      for (int ky = 0; ky < k; ++ky) {
        const int y = yy - ky + p;
        if (y < 0 || y >= h) continue;
        for (int kx = 0; kx < k; ++kx) {
          const int x = xx - kx + p;
          if (x < 0 || x >= w) continue;
          s += *reinterpret_cast<const f32x4 *>(dP + ((b * h + y) * w + x) * (int64_t)kkc + (ky * k + kx) * c + ch);
        }
      }
      *reinterpret_cast<f32x4 *>(din + 4 * i) = s;
    }
    return;
  }
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += step) {
    const int ch = (int)(i % c);
    int64_t r = i / c;
    const int xx = (int)(r % w);
    r /= w;
    const int yy = (int)(r % h);
    const int64_t b = r / h;
    float s = 0.f;
    for (int ky = 0; ky < k; ++ky) {
      const int y = yy - ky + p;
      if (y < 0 || y >= h) continue;
      for (int kx = 0; kx < k; ++kx) {
        const int x = xx - kx + p;
        if (x < 0 || x >= w) continue;
        s += dP[((b * h + y) * w + x) * (int64_t)kkc + (ky * k + kx) * c + ch];
      }
    }
    din[i] = s;
  }
}


// ---- a conv block with FEW input values per output (first layers on images: one or a few ----
// channels, a small filter): forward product, relu and 2 x 2 pooling in one kernel, no patch
// matrix and no pre-activation in memory.  A workgroup takes a band of pooled rows of one example:
// the zero-padded band of the image and the whole filter bank sit in LDS, a work item is one pooled
// cell and four filters (its four window positions, 16 sums, each over the taps in the order
// (dy, dx, channel) of the filter layout).  Output as relu_pool_kernel writes it.
constexpr int kDirectWeights = 4096;   // floats of LDS for the filter bank
constexpr int kDirectPatch = 4096;     // floats of LDS for the padded band of the image
constexpr int kDirectTaps = 56;        // k k c_in up to this: from 64 taps on the matrix cores win

__global__ __launch_bounds__(kThreads) void conv_relu_pool_kernel(const float *in, const float *Wc,
                                                                  const float *bias, int h, int w, int ci, int k,
                                                                  int co, int band, float *pooled,
                                                                  uint8_t *which) {
  __shared__ __align__(16) float wts[kDirectWeights];
  __shared__ float patch[kDirectPatch];
  const int p = (k - 1) / 2, ho = h / 2, wo = w / 2, kkc = k * k * ci;
  const int bands = (ho + band - 1) / band;
  const int64_t b = blockIdx.x / bands;
  const int yo0 = (int)(blockIdx.x % bands) * band;
  const int rows_o = min(band, ho - yo0);
  const int pr = 2 * rows_o + k - 1, pw = w + k - 1, pwc = pw * ci;   // the padded band: rows, columns
  for (int i = threadIdx.x; i < kkc * co / 4; i += kThreads)
    reinterpret_cast<f32x4 *>(wts)[i] = reinterpret_cast<const f32x4 *>(Wc)[i];
  const float *src = in + b * h * w * ci;
  for (int i = threadIdx.x; i < pr * pwc; i += kThreads) {
    const int r = i / pwc, rem = i - r * pwc, q = rem / ci;
    const int y = 2 * yo0 - p + r, x = q - p;
    patch[i] = (y >= 0 && y < h && x >= 0 && x < w) ? src[(y * w + x) * ci + (rem - q * ci)] : 0.f;
  }
  __syncthreads();
  const int co4 = co / 4, kc = k * ci;
  const int items = rows_o * wo * co4;
  for (int it = threadIdx.x; it < items; it += kThreads) {
    const int fq = it % co4, cell = it / co4;
    const int yl = cell / wo, xo = cell - yl * wo;
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    const f32x4 bv = bias ? *reinterpret_cast<const f32x4 *>(bias + 4 * fq) : zero;
    f32x4 acc[4] = {bv, bv, bv, bv};
    // tap (dy, dx, c) of window position (py, px): patch row 2 yl + py + dy, column 2 xo + px + dx;
    // for one dy the offsets dx ci + c run through 0 .. k ci - 1, and so do the filter's rows
    const float *origin = patch + (2 * yl * pw + 2 * xo) * ci;
    const float *wp = wts + 4 * fq;
    for (int dy = 0; dy < k; ++dy) {
      const float *q0 = origin + dy * pwc;
      const float *wrow = wp + dy * kc * co;
#pragma unroll 5
      for (int t = 0; t < kc; ++t) {
        const f32x4 wv = *reinterpret_cast<const f32x4 *>(wrow + t * co);
        const float v00 = q0[t], v01 = q0[t + ci], v10 = q0[t + pwc], v11 = q0[t + pwc + ci];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          acc[0][q] = fmaf(v00, wv[q], acc[0][q]);
          acc[1][q] = fmaf(v01, wv[q], acc[1][q]);
          acc[2][q] = fmaf(v10, wv[q], acc[2][q]);
          acc[3][q] = fmaf(v11, wv[q], acc[3][q]);
        }
      }
    }
    f32x4 best = {-1.f, -1.f, -1.f, -1.f};
    uint32_t arg = 0;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float a = acc[d][q] > 0.f ? acc[d][q] : 0.f;
        if (a > best[q]) {
          best[q] = a;
          arg = (arg & ~(0xffu << (8 * q))) | ((uint32_t)d << (8 * q));
        }
      }
    }
    const int64_t group = ((b * ho + yo0 + yl) * wo + xo) * co4 + fq;   // four channels of a pooled cell
    *reinterpret_cast<f32x4 *>(pooled + 4 * group) = best;
    *reinterpret_cast<uint32_t *>(which + 4 * group) = arg;
  }
}

// pooled rows per workgroup: about 1024 workgroups over the batch (measured best of 256 .. 2048), a band that fits the LDS buffer
// (0: none does)
int direct_band(int64_t B, int h, int w, int ci, int k) {
  const int ho = h / 2;
  const int64_t per_example = std::max<int64_t>(1, std::min<int64_t>(ho, (1024 + B - 1) / B));
  int band = (int)((ho + per_example - 1) / per_example);
  const int64_t pwc = (int64_t)(w + k - 1) * ci;
  while (band > 1 && (2 * band + k - 1) * pwc > kDirectPatch) --band;
  return (2 * band + k - 1) * pwc > kDirectPatch ? 0 : band;
}

}  // namespace

hipError_t launch_im2col(const float *in, int64_t B, int32_t h, int32_t w, int32_t c, int32_t k,
                         float *P, float *PT, hipStream_t stream) {
  const int64_t hw = (int64_t)h * w, kkc = (int64_t)k * k * c;
  if (B <= 0 || hw <= 0 || kkc <= 0) return hipSuccess;
  if (B > 65535) return hipErrorInvalidValue;
  auto aligned = [](const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15) == 0; };
  if (c % 4 != 0 && hw * c <= kLdsImage && (hw * kkc) % 4 == 0 && hw * kkc < (1 << 24) && aligned(P) && aligned(PT)) {
    // enough workgroups for the chip, slabs of at least 1024 values
    int64_t slabs = (1024 + B - 1) / B;
    slabs = std::max<int64_t>(1, std::min<int64_t>(slabs, hw * kkc / 1024));
    PFG_KERNEL(im2col_lds_kernel, dim3((unsigned)slabs, (unsigned)B), dim3(kThreads), 0, stream, in, h, w, c, k,
               P, PT);
    return hipGetLastError();
  }
  if (P) {
    if (c % 4 != 0 && (reinterpret_cast<uintptr_t>(P) & 15) == 0)
      PFG_KERNEL(im2col_flat_kernel, dim3(capped_blocks((B * hw * kkc + 3) / 4)), dim3(kThreads), 0, stream, in,
                 B, h, w, c, k, P);
    else
      PFG_KERNEL(im2col_kernel<true>, dim3((unsigned)((hw + kRows - 1) / kRows), (unsigned)B), dim3(kThreads),
                 0, stream, in, h, w, c, k, P);
  }
  if (PT) {
    const int64_t runs = (hw + kPosRun - 1) / kPosRun;
    if (c >= 8 && c <= kMaxTiledC && runs <= 65535)
      PFG_KERNEL(im2col_pt_tiled_kernel, dim3((unsigned)(k * k), (unsigned)runs, (unsigned)B), dim3(kThreads), 0,
                 stream, in, h, w, c, k, PT);
    else
      PFG_KERNEL(im2col_kernel<false>, dim3((unsigned)((kkc + kRows - 1) / kRows), (unsigned)B),
                 dim3(kThreads), 0, stream, in, h, w, c, k, PT);
  }
  return hipGetLastError();
}

hipError_t launch_relu_pool(const float *z, int64_t B, int32_t h, int32_t w, int32_t c, float *pooled,
                            uint8_t *which, hipStream_t stream) {
  const int64_t total = B * (h / 2) * (w / 2) * c;
  if (total <= 0) return hipSuccess;
  PFG_KERNEL(relu_pool_kernel, dim3(capped_blocks(total)), dim3(kThreads), 0, stream, z, B, h, w, c,
             pooled, which);
  return hipGetLastError();
}

bool conv_relu_pool_applies(const float *in, const float *Wc, const float *bias, int64_t B, int32_t h, int32_t w,
                            int32_t ci, int32_t k, int32_t co, const float *pooled, const uint8_t *which) {
  if (!in || !Wc || !pooled || !which || B < 1 || h < 2 || w < 2 || h % 2 || w % 2) return false;
  const int64_t kkc = (int64_t)k * k * ci;
  if (co % 4 != 0 || kkc > kDirectTaps || kkc * co > kDirectWeights) return false;
  const int band = direct_band(B, h, w, ci, k);
  if (band < 1 || B * ((h / 2 + band - 1) / band) > 0x7fffffffLL) return false;
  return (reinterpret_cast<uintptr_t>(which) & 3) == 0 &&
         ((reinterpret_cast<uintptr_t>(Wc) | reinterpret_cast<uintptr_t>(bias) |
           reinterpret_cast<uintptr_t>(pooled)) & 15) == 0;
}

hipError_t launch_conv_relu_pool(const float *in, const float *Wc, const float *bias, int64_t B, int32_t h,
                                 int32_t w, int32_t ci, int32_t k, int32_t co, float *pooled, uint8_t *which,
                                 hipStream_t stream) {
  if (!conv_relu_pool_applies(in, Wc, bias, B, h, w, ci, k, co, pooled, which)) return hipErrorInvalidValue;
  const int band = direct_band(B, h, w, ci, k);
  const int64_t bands = (h / 2 + band - 1) / band;
  PFG_KERNEL(conv_relu_pool_kernel, dim3((unsigned)(B * bands)), dim3(kThreads), 0, stream, in, Wc, bias, h, w,
             ci, k, co, band, pooled, which);
  return hipGetLastError();
}

hipError_t launch_unpool_mask(const float *dpooled, const float *pooled, const uint8_t *which, int64_t B,
                              int32_t h, int32_t w, int32_t c, float *dz, hipStream_t stream) {
  const int64_t total = B * (h / 2) * (w / 2) * c;
  if (total <= 0) return hipSuccess;
  PFG_KERNEL(unpool_mask_kernel, dim3(capped_blocks(total)), dim3(kThreads), 0, stream, dpooled, pooled,
             which, B, h, w, c, dz);
  return hipGetLastError();
}

bool unpool_mask_sum_applies(const float *dpooled, const float *pooled, const uint8_t *which, int64_t B,
                             int32_t h, int32_t w, int32_t c, const float *dz, const float *db) {
  // a workgroup per example: worth it once the examples alone give the chip enough workgroups
  if (B < 32 || B > 0x7fffffffLL || c % 4 != 0 || c > 4 * kThreads) return false;
  if ((int64_t)(h / 2) * (w / 2) * (c / 4) > 0x7fffffffLL) return false;
  return (reinterpret_cast<uintptr_t>(which) & 3) == 0 &&
         ((reinterpret_cast<uintptr_t>(dpooled) | reinterpret_cast<uintptr_t>(pooled) |
           reinterpret_cast<uintptr_t>(dz) | reinterpret_cast<uintptr_t>(db)) & 15) == 0;
}

hipError_t launch_unpool_mask_sum(const float *dpooled, const float *pooled, const uint8_t *which, int64_t B,
                                  int32_t h, int32_t w, int32_t c, float *dz, float *db, hipStream_t stream) {
  if (B <= 0 || (int64_t)(h / 2) * (w / 2) * c <= 0) return hipSuccess;
  if (!unpool_mask_sum_applies(dpooled, pooled, which, B, h, w, c, dz, db)) return hipErrorInvalidValue;
  PFG_KERNEL(unpool_mask_sum_kernel, dim3((unsigned)B), dim3(kThreads), 0, stream, dpooled, pooled, which,
             h, w, c, dz, db);
  return hipGetLastError();
}

hipError_t launch_col2im(const float *dP, int64_t B, int32_t h, int32_t w, int32_t c, int32_t k,
                         float *din, hipStream_t stream) {
  const int64_t total = B * h * w * c;
  if (total <= 0) return hipSuccess;
  PFG_KERNEL(col2im_kernel, dim3(capped_blocks(total)), dim3(kThreads), 0, stream, dP, B, h, w, c, k, din);
  return hipGetLastError();
}

}  // namespace pfg
