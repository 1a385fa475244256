// Small row-wise and element-wise kernels: the loss head, the seed rows of the Jacobians, a
// transpose, activation derivatives from stored pre-activations, row scaling, and the squared
// norms of rank-one gradients.
// Each row is handled by one 64-lane wave; lanes stride over the d_L classes and combine with
// wave reductions (Section 3.4: a reduction inside the loop body keeps reducing over its own
// axis after vectorisation; it never reduces over the iteration index).
#include "common.h"
#include "gemm_device.h"

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

// a = phi(z), dphi = phi'(z), d2phi = phi''(z), element by element.
__global__ __launch_bounds__(kThreads) void act_from_z_kernel(const float *z, int64_t n, int act,
                                                              float *a, float *dphi, float *d2phi) {
  const int64_t step = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += step) {
    const float v = z[i];
    if (a) a[i] = dev::act_value(act, v);
    if (dphi) dphi[i] = dev::act_deriv(act, v);
    if (d2phi) d2phi[i] = dev::act_deriv2(act, v);
  }
}

// Second half of a product whose contraction was cut into Z pieces (see launch_gemm_split): adds
// the Z partial results [Z, M, N] in a fixed order and applies the epilogue of the whole product.
__global__ __launch_bounds__(kThreads) void split_finish_kernel(const float *part, int Z, int64_t mn, int N,
                                                                const void *bias, int bias_bf16, int epilogue,
                                                                int act, float *C, float *C2, int64_t ldc) {
  const int64_t step = (int64_t)gridDim.x * kThreads;
  for (int64_t q = (int64_t)blockIdx.x * kThreads + threadIdx.x; q < mn / 4; q += step) {
    const int64_t i = 4 * q;
    const int64_t m = i / N;
    const int n = (int)(i - m * N);
    f32x4 v = *reinterpret_cast<const f32x4 *>(part + i);
    for (int z = 1; z < Z; ++z) v += *reinterpret_cast<const f32x4 *>(part + z * mn + i);
    if (bias && epilogue != EPI_NONE) {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        v[e] += bias_bf16 ? (float)static_cast<const __bf16 *>(bias)[n + e] : static_cast<const float *>(bias)[n + e];
    }
    f32x4 out = v, out2 = v;
    if (epilogue == EPI_FORWARD) {
#pragma unroll
      for (int e = 0; e < 4; ++e) { out[e] = dev::act_value(act, v[e]); out2[e] = dev::act_deriv(act, v[e]); }
    }
    if (C) *reinterpret_cast<f32x4 *>(C + m * ldc + n) = out;
    if (C2 && epilogue == EPI_FORWARD) *reinterpret_cast<f32x4 *>(C2 + m * ldc + n) = out2;
  }
}

// out[(b, s), j] = in[b, s, j] * mask[b, j]: the mask of a layer does not depend on the inner
// iteration index s and is broadcast over it (Section 3.4: loop-invariant operands are not stacked).
__global__ __launch_bounds__(kThreads) void scale_rows_kernel(const void *in, int in_bf16,
                                                              int64_t in_batch_stride, int64_t ld_in,
                                                              const float *mask, int64_t ld_mask,
                                                              int64_t rows, int64_t S, int d,
                                                              float *out, int64_t ld_out) {
  const int64_t total = rows * d;
  const int64_t step = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += step) {
    const int64_t row = i / d;
    const int j = (int)(i - row * d);
    const int64_t b = row / S, s = row - b * S;
    const int64_t at = b * in_batch_stride + s * ld_in + j;
    float v = in_bf16 ? (float)static_cast<const __bf16 *>(in)[at] : static_cast<const float *>(in)[at];
    if (mask) v *= mask[b * ld_mask + j];
    out[row * ld_out + j] = v;
  }
}

// This thread's share of the sum of squares of one float32 row (16-byte loads when the row allows).
__device__ __forceinline__ float row_sumsq(const float *row, int d, int tid) {
  float s = 0.f;
  if ((reinterpret_cast<uintptr_t>(row) & 15) == 0 && d % 4 == 0) {
    const f32x4 *r4 = reinterpret_cast<const f32x4 *>(row);
    const int n4 = d / 4;
    int i = tid;
    // long rows: four loads in flight per thread, four partial sums folded in a fixed order
    float s1 = 0.f, s2 = 0.f, s3 = 0.f;
    for (; i + 3 * kThreads < n4; i += 4 * kThreads) {
      const f32x4 v0 = r4[i], v1 = r4[i + kThreads], v2 = r4[i + 2 * kThreads], v3 = r4[i + 3 * kThreads];
      s += v0[0] * v0[0] + v0[1] * v0[1] + v0[2] * v0[2] + v0[3] * v0[3];
      s1 += v1[0] * v1[0] + v1[1] * v1[1] + v1[2] * v1[2] + v1[3] * v1[3];
      s2 += v2[0] * v2[0] + v2[1] * v2[1] + v2[2] * v2[2] + v2[3] * v2[3];
      s3 += v3[0] * v3[0] + v3[1] * v3[1] + v3[2] * v3[2] + v3[3] * v3[3];
    }
    s = (s + s1) + (s2 + s3);
    for (; i < n4; i += kThreads) {
      const f32x4 v = r4[i];
      s += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
    }
  } else {
    for (int i = tid; i < d; i += kThreads) { const float v = row[i]; s += v * v; }
  }
  return s;
}

struct NormBatch {
  NormLayer layer[kNormLayers];
  int n;
};

// The gradient of a dense layer for one example is the outer product of the layer's input row and
// its cotangent row (the both-operands-stacked matmul case of Section 3.4 with contraction
// length 1), so its squared Frobenius norm is the product of the two rows' squared norms; the
// bias gradient is the cotangent row itself.  A block whose gradient has been formed (sum_mode: a
// convolution's filter, summed over the positions) contributes the sum of its squares instead
// (sum_mode 1), or partial sums of those squares that the kernel forming it left behind (sum_mode 2).
// One workgroup per example, sums in a fixed order.
__global__ __launch_bounds__(kThreads) void grad_sqnorms_kernel(const NormBatch nb, float *sq,
                                                                int64_t ld_sq, float *norm) {
  __shared__ float part[2][kWavesPerBlock];
  const int64_t b = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float total = 0.f;
  for (int li = 0; li < nb.n; ++li) {
    const NormLayer &ly = nb.layer[li];
    float sa = 0.f, sg = 0.f;
    if (ly.sum_mode == 2) {
      // the block's squares were summed where its gradient was formed: d_in partial sums per example
      const float *a = static_cast<const float *>(ly.a) + b * ly.d_in;
      for (int i = tid; i < ly.d_in; i += kThreads) sa += a[i];
    } else if (ly.a_bf16) {
      const __bf16 *a = static_cast<const __bf16 *>(ly.a) + b * ly.d_in;
      for (int i = tid; i < ly.d_in; i += kThreads) { const float v = (float)a[i]; sa += v * v; }
    } else {
      sa = row_sumsq(static_cast<const float *>(ly.a) + b * ly.d_in, ly.d_in, tid);
    }
    if (ly.g) sg = row_sumsq(ly.g + b * ly.d_out, ly.d_out, tid);
    sa = wave_sum(sa);
    sg = wave_sum(sg);
    __syncthreads();                       // the previous layer's partial sums have been read
    if (lane == 0) { part[0][wave] = sa; part[1][wave] = sg; }
    __syncthreads();
    float ta = 0.f, tg = 0.f;
#pragma unroll
    for (int w = 0; w < kWavesPerBlock; ++w) { ta += part[0][w]; tg += part[1][w]; }
    const float v = ly.sum_mode ? ta + tg : (ta + (ly.has_bias ? 1.f : 0.f)) * tg;
    if (sq && tid == 0) sq[b * ld_sq + ly.index] = v;
    total += v;
  }
  if (norm && tid == 0) norm[b] = sqrtf(total);
}

__global__ __launch_bounds__(kThreads) void norm_finalize_kernel(const float *sq, int64_t ld_sq, int L,
                                                                 int64_t B, float *norm) {
  const int64_t b = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (b >= B) return;
  float total = 0.f;
  for (int l = 0; l < L; ++l) total += sq[b * ld_sq + l];
  norm[b] = sqrtf(total);
}

__global__ __launch_bounds__(kThreads) void fill_zero_kernel(float *out, int64_t n) {
  const int64_t step = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += step) out[i] = 0.f;
}

// The stitching step after a loop with a shrinking set of active iterations (Section 3.7): row j
// of the compacted state goes back to the slot of the iteration it belongs to.
__global__ __launch_bounds__(kThreads) void scatter_rows_kernel(const float *src_even, const float *src_odd,
                                                                const int32_t *parity,
                                                                const int32_t *order, int64_t rows,
                                                                int d, float *out) {
  const int64_t total = rows * d;
  const int64_t step = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += step) {
    const int64_t j = i / d;
    const int k = (int)(i - j * d);
    const float *src = (parity[j] & 1) ? src_odd : src_even;
    out[(int64_t)order[j] * d + k] = src[j * d + k];
  }
}

inline unsigned capped_blocks(int64_t work_items) {
  const int64_t blocks = (work_items + kThreads - 1) / kThreads;
  return (unsigned)(blocks < (1 << 20) ? blocks : (1 << 20));
}

}  // namespace

hipError_t launch_act_from_z(const float *z, int64_t B, int32_t d, int32_t act, float *a, float *dphi,
                             float *d2phi, hipStream_t stream) {
  const int64_t n = B * d;
  if (n <= 0) return hipSuccess;
  PFG_KERNEL(act_from_z_kernel, dim3(capped_blocks(n)), dim3(kThreads), 0, stream, z, n, act, a, dphi,
             d2phi);
  return hipGetLastError();
}

hipError_t launch_scale_rows(const void *in, int32_t in_bf16, int64_t in_batch_stride, int64_t ld_in,
                             const float *mask, int64_t ld_mask, int64_t B, int64_t S, int32_t d,
                             float *out, int64_t ld_out, hipStream_t stream) {
  const int64_t rows = B * S;
  if (rows <= 0 || d <= 0) return hipSuccess;
  PFG_KERNEL(scale_rows_kernel, dim3(capped_blocks(rows * d)), dim3(kThreads), 0, stream, in, in_bf16,
             in_batch_stride, ld_in, mask, ld_mask, rows, S, d, out, ld_out);
  return hipGetLastError();
}

int split_k_factor(const GemmArgs &g) {
  auto aligned = [](const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15) == 0; };
  if (g.a_scale || g.nbatch > 1 || g.sub || g.sym_n > 0 || g.a_km || g.S != 1) return 1;
  if (!g.bf16 && !g.a_is_f32) return 1;
  if (g.epilogue != EPI_NONE && g.epilogue != EPI_BIAS && g.epilogue != EPI_FORWARD) return 1;
  if (!g.w_kn) return 1;       // weights in [N, K] layout (cotangent steps): measured no faster when cut
  if (g.ldc % 4 || g.lda % 8 || g.ldw % 8) return 1;
  if (!aligned(g.A) || !aligned(g.W) || (g.C && !aligned(g.C)) || (g.C2 && !aligned(g.C2))) return 1;
  return split_k_shape(g.M, g.N, g.K, g.bf16);
}

int split_k_shape(int64_t M, int64_t N, int64_t K, int bf16) {
  // fewer than 64 rows: measured a gain for bf16 weights only (4096 x 4096 at 8 to 48 rows: 55 -> 30 us
  // per product; a float32 3136 x 1024 layer got 5 us slower)
  if (M < (bf16 ? 1 : 64) || N < 256 || N % 8 || K < 1024) return 1;
  const int64_t tiles64 = ((M + 63) / 64) * ((N + 63) / 64);
  if (tiles64 < 128) {
    // too few tiles for the chip: up to 8 pieces of at least 256, if that makes 128 workgroups or
    // more (with fewer the small-problem kernels are the better choice: 64 rows against
    // 1024 x 1024 weights took 25 us in four pieces on 64 workgroups, 15 us there)
    for (int Z = 8; Z >= 2; Z /= 2)
      if (K % (8 * Z) == 0 && K / Z >= 256 && Z * tiles64 <= 512 && Z * tiles64 >= 128) return Z;
    return 1;
  }
  // 128 to 256 tiles: the tiled kernel would run one workgroup on some or all of the 256 units.
  // bf16 products are then bound by the instruction issue of a single wave per SIMD, float32
  // products leave units idle; two pieces give every unit two workgroups.  (float32 products of
  // 128 to 191 tiles go to the small-problem kernels instead, see launch_gemm.)
  if (bf16) return (tiles64 <= 256 && K >= 2048 && K % 128 == 0) ? 2 : 1;
  return (tiles64 >= 192 && tiles64 < 256 && K % 16 == 0) ? 2 : 1;
}

hipError_t launch_gemm_split(const GemmArgs &g, int Z, float *partials, hipStream_t stream) {
  if (Z < 2 || Z != split_k_factor(g) || !partials) return hipErrorInvalidValue;
  const int Kz = g.K / Z;
  GemmArgs b = g;
  b.K = Kz;
  b.nbatch = Z;
  b.batch_A = Kz;                                       // piece z: columns z Kz .. of A,
  b.batch_W = (int64_t)Kz * g.ldw;                      // rows z Kz .. of W [K, N]
  b.batch_C = (int64_t)g.M * g.N;
  b.C = partials; b.ldc = g.N; b.C2 = nullptr;
  b.epilogue = EPI_NONE; b.bias = nullptr; b.streaming = 0;
  hipError_t e = launch_gemm(b, stream);
  if (e != hipSuccess) return e;
  const int64_t mn = (int64_t)g.M * g.N;
  PFG_KERNEL(split_finish_kernel, dim3(capped_blocks(mn / 4)), dim3(kThreads), 0, stream, partials, Z, mn, g.N,
             g.bias, g.bf16, g.epilogue, g.act, g.C, g.C2, g.ldc);
  return hipGetLastError();
}

hipError_t launch_grad_sqnorms(const NormLayer *layers, int n, int64_t B, float *sq, int64_t ld_sq,
                               float *norm, hipStream_t stream) {
  if (B <= 0 || n <= 0) return hipSuccess;
  if (n > kNormLayers || B > 0x7fffffffLL) return hipErrorInvalidValue;
  NormBatch nb{};
  for (int i = 0; i < n; ++i) nb.layer[i] = layers[i];
  nb.n = n;
  PFG_KERNEL(grad_sqnorms_kernel, dim3((unsigned)B), dim3(kThreads), 0, stream, nb, sq, ld_sq, norm);
  return hipGetLastError();
}

hipError_t launch_norm_finalize(const float *sq, int64_t ld_sq, int32_t L, int64_t B, float *norm,
                                hipStream_t stream) {
  if (B <= 0) return hipSuccess;
  PFG_KERNEL(norm_finalize_kernel, dim3((unsigned)((B + kThreads - 1) / kThreads)), dim3(kThreads), 0,
             stream, sq, ld_sq, L, B, norm);
  return hipGetLastError();
}

hipError_t launch_scatter_rows(const float *src_even, const float *src_odd, const int32_t *parity,
                               const int32_t *order, int64_t rows, int32_t d, float *out,
                               hipStream_t stream) {
  if (rows <= 0 || d <= 0) return hipSuccess;
  PFG_KERNEL(scatter_rows_kernel, dim3(capped_blocks(rows * d)), dim3(kThreads), 0, stream, src_even,
             src_odd, parity, order, rows, d, out);
  return hipGetLastError();
}

hipError_t launch_fill_zero(float *out, int64_t n, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  PFG_KERNEL(fill_zero_kernel, dim3(capped_blocks(n)), dim3(kThreads), 0, stream, out, n);
  return hipGetLastError();
}

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
