// Loss head for a last layer with a LONG contraction and few rows.
//
// The fused head of the small-problem kernel computes the logits of a 32-row tile in every
// workgroup that shares the tile's cotangent step; with d_{L-1} in the thousands each of them
// streams its rows over the whole contraction, and that dominates.  Here the logits are computed
// once, as Z partial products over pieces of the contraction (one batch entry of the tiled product
// kernel each), and this kernel does the rest for a tile: it adds the partial logits in a fixed
// order, then softmax cross-entropy (loss and delta_L), then its share of the cotangent step
// through the last layer.  Same arithmetic as the fused head, another order of summation.
#include "common.h"
#include "gemm_device.h"

namespace pfg {

namespace {

using namespace dev;

constexpr int kHeadThreads = 256;

// partials [Z, M, N]; the remaining arguments as for EPI_HEAD (GemmArgs: M, N, K, W, ldw, bf16, bias,
// labels, loss, C2 = delta [M, ldc], head_gprev / head_mask [M, K]).  Grid: row tiles of 32 times
// the workgroups that share a tile's cotangent step.
__global__ __launch_bounds__(kHeadThreads) void head_from_partials_kernel(const GemmArgs g,
                                                                          const float *partials, int Z) {
  __shared__ float y[32][33];
  __shared__ float yh[2][32 * 32];        // the two halves of the pieces, added separately first
  __shared__ __align__(16) float hd[32][32];
  __shared__ int lab[32];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int half = lane >> 5, l32 = lane & 31;
  const int N = g.N, M = g.M;
  const int tiles_m = (M + 31) / 32;
  const int m0 = (blockIdx.x % tiles_m) * 32;
  const int second = blockIdx.x / tiles_m;
  const int tile_rows = min(32, M - m0);
  if (tid < 32) lab[tid] = (tid < tile_rows) ? g.labels[m0 + tid] : -1;
  // logits of the tile: bias plus the partial products.  A work item is (element, half of the
  // pieces) with up to 16 loads in flight at once; the halves are then
  // added in a fixed order.
  const int64_t mn = (int64_t)M * N;
  const int items = tile_rows * N, zh = (Z + 1) / 2;
  for (int w = tid; w < 2 * items; w += kHeadThreads) {
    const int hf = w / items, e = w - hf * items;
    const int row = e / N, col = e - row * N;
    const float *p = partials + (int64_t)(m0 + row) * N + col;
    const int z_begin = hf * zh, z_end = min(Z, z_begin + zh);
    float v = 0.f;
    for (int z0 = z_begin; z0 < z_end; z0 += 16) {
      float t[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) t[u] = (z0 + u < z_end) ? p[(z0 + u) * mn] : 0.f;
#pragma unroll
      for (int u = 0; u < 16; ++u) v += t[u];
    }
    yh[hf][e] = v;
  }
  __syncthreads();
  for (int e = tid; e < items; e += kHeadThreads) {
    const int row = e / N, col = e - row * N;
    float v = yh[0][e] + yh[1][e];
    if (g.bias) v += g.bf16 ? (float)static_cast<const __bf16 *>(g.bias)[col] : static_cast<const float *>(g.bias)[col];
    y[row][col] = v;
  }
  __syncthreads();
  // softmax cross-entropy: each half of a wave takes one row per pass (N <= 32)
#pragma unroll 1
  for (int row0 = 2 * wave; row0 < 32; row0 += 2 * (kHeadThreads / 64)) {
    const int row = row0 + half;
    const int m = m0 + row;
    const bool valid = row < tile_rows;
    const bool live = valid && (l32 < N);
    const float yv = live ? y[row][l32] : -INFINITY;
    float mx = yv;
#pragma unroll
    for (int off = 16; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    const float ex = live ? __expf(yv - mx) : 0.f;
    const int label = lab[row];
    float den = ex, others = (l32 == label) ? 0.f : ex;
#pragma unroll
    for (int off = 16; off > 0; off >>= 1) {
      den += __shfl_xor(den, off, 64);
      others += __shfl_xor(others, off, 64);
    }
    const float inv = valid ? 1.f / den : 0.f;
    // p[label] - 1 = -(sum of the other classes) / den, free of cancellation
    const float delta = (l32 == label) ? -others * inv : ex * inv;
    if (live && second == 0) g.C2[(int64_t)m * g.ldc + l32] = delta;
    hd[row][l32] = live ? delta : 0.f;
    const bool label_ok = (label >= 0) && (label < N);
    const float yl = __shfl(yv, half * 32 + (label_ok ? label : 0), 64);
    if (g.loss && valid && l32 == 0 && second == 0) g.loss[m] = __logf(den) - ((label_ok ? yl : mx) - mx);
  }
  if (!g.head_gprev) return;
  __syncthreads();
  const int groups = (int)gridDim.x / tiles_m;
  switch ((N + 3) >> 2) {
    case 1: head_cotangent<1, kHeadThreads, 4>(g, hd, m0, tile_rows, tid, second, groups); break;
    case 2: head_cotangent<2, kHeadThreads, 4>(g, hd, m0, tile_rows, tid, second, groups); break;
    case 3: head_cotangent<3, kHeadThreads, 4>(g, hd, m0, tile_rows, tid, second, groups); break;
    case 4: head_cotangent<4, kHeadThreads, 4>(g, hd, m0, tile_rows, tid, second, groups); break;
    case 5: head_cotangent<5, kHeadThreads, 4>(g, hd, m0, tile_rows, tid, second, groups); break;
    case 6: head_cotangent<6, kHeadThreads, 4>(g, hd, m0, tile_rows, tid, second, groups); break;
    case 7: head_cotangent<7, kHeadThreads, 4>(g, hd, m0, tile_rows, tid, second, groups); break;
    default: head_cotangent<8, kHeadThreads, 4>(g, hd, m0, tile_rows, tid, second, groups); break;
  }
}

// ------------------------------------------------------------------------------------------
// Loss head of a NARROW network with few rows: one workgroup per example.
//
// The last layer has at most 16 outputs and its input at most 1024 units: thread t then keeps the
// rows t, t + 256, ... of W_L (CPT of them, N floats each) in registers and uses them twice -- for
// its share of the logits (joined through LDS in a fixed order) and, after the softmax, for its
// columns of the cotangent step through the same layer.  One pass over global memory, one
// launch, where the fused head of the small-problem kernel walks three dependent phases
// (11.7 -> 4.5 us at 128 rows, 512 units, 10 classes).
//   mode 0 (per-example gradients): delta = softmax(y) - onehot(label) -> C2 [M, ldc], loss,
//           head_gprev[m, i] = head_mask[m, i] * sum_j delta[j] W[i, j]
//   mode 1 (Jacobian of softmax(y), identity seeds, S = N rows per example):
//           G_L[m, k, j] = p_k (delta_kj - p_j)                          -> C2 [M * N, ldc]
//           G_prev[m, k, i] = head_mask[m, i] p_k (W[i, k] - sum_j p_j W[i, j])   -> head_gprev [M * N, K]
// ------------------------------------------------------------------------------------------
constexpr int kRowsMaxN = 16;

template <int CPT>
__global__ __launch_bounds__(kHeadThreads) void head_rows_kernel(const GemmArgs g, int mode) {
  __shared__ float part[kRowsMaxN][kHeadThreads + 4];
  __shared__ float part2[kRowsMaxN][16];
  __shared__ float ys[kRowsMaxN];
  const int tid = threadIdx.x;
  const int64_t m = blockIdx.x;
  const int N = g.N, K = g.K;
  const float *W = static_cast<const float *>(g.W);
  const float *arow = static_cast<const float *>(g.A) + m * g.lda;
  // this thread's rows of W and entries of a, requested at once
  float w[CPT][kRowsMaxN], a[CPT], mask[CPT];
#pragma unroll
  for (int c = 0; c < CPT; ++c) {
    const int i = tid + c * kHeadThreads;
    const bool in = i < K;
    a[c] = in ? arow[i] : 0.f;
    mask[c] = (in && g.head_gprev) ? g.head_mask[m * K + i] : 0.f;
#pragma unroll
    for (int j = 0; j < kRowsMaxN; ++j) w[c][j] = (in && j < N) ? W[(int64_t)i * g.ldw + j] : 0.f;
  }
  const int label = (mode == 0) ? g.labels[m] : -1;
  // partial logits of this thread, then a fixed-order sum: 16 segments of 16 threads, then the segments
#pragma unroll
  for (int j = 0; j < kRowsMaxN; ++j) {
    float v = 0.f;
#pragma unroll
    for (int c = 0; c < CPT; ++c) v += a[c] * w[c][j];
    part[j][tid] = v;
  }
  __syncthreads();
  {
    const int j = tid >> 4, seg = tid & 15;
    float v = 0.f;
#pragma unroll
    for (int u = 0; u < 16; ++u) v += part[j][seg * 16 + u];
    part2[j][seg] = v;
  }
  __syncthreads();
  if (tid < kRowsMaxN) {
    float v = 0.f;
#pragma unroll
    for (int u = 0; u < 16; ++u) v += part2[tid][u];
    if (tid < N && g.bias) v += static_cast<const float *>(g.bias)[tid];
    ys[tid] = v;
  }
  __syncthreads();
  // softmax of the row (every thread, from LDS: N <= 16 values)
  float pr[kRowsMaxN];
  float mx = -INFINITY;
#pragma unroll
  for (int j = 0; j < kRowsMaxN; ++j) {
    pr[j] = j < N ? ys[j] : -INFINITY;
    mx = fmaxf(mx, pr[j]);
  }
  float den = 0.f, others = 0.f, ylab = mx;
#pragma unroll
  for (int j = 0; j < kRowsMaxN; ++j) {
    if (j == label) ylab = pr[j];
    pr[j] = j < N ? __expf(pr[j] - mx) : 0.f;
    den += pr[j];
    if (j != label) others += pr[j];
  }
  const float inv = 1.f / den;
  if (mode == 0) {
    // delta = p - onehot; the label's entry as -(sum of the others) / den, free of cancellation
#pragma unroll
    for (int j = 0; j < kRowsMaxN; ++j) pr[j] = (j == label) ? -others * inv : pr[j] * inv;
    if (tid < N) {
      float d = 0.f;
#pragma unroll
      for (int j = 0; j < kRowsMaxN; ++j)
        if (j == tid) d = pr[j];
      g.C2[m * g.ldc + tid] = d;
    }
    if (tid == 0 && g.loss) g.loss[m] = __logf(den) - (ylab - mx);
    if (g.head_gprev) {
#pragma unroll
      for (int c = 0; c < CPT; ++c) {
        const int i = tid + c * kHeadThreads;
        float v = 0.f;
#pragma unroll
        for (int j = 0; j < kRowsMaxN; ++j) v += pr[j] * w[c][j];
        if (i < K) g.head_gprev[m * K + i] = v * mask[c];
      }
    }
    return;
  }
  // mode 1: the N rows d softmax(y)_k / d y = p_k (e_k - p), and their pull-back through W
#pragma unroll
  for (int j = 0; j < kRowsMaxN; ++j) pr[j] *= inv;
  if (g.C2 && tid < N * N) {
    const int k = tid / N, j = tid - k * N;
    float pk = 0.f, pj = 0.f;
#pragma unroll
    for (int u = 0; u < kRowsMaxN; ++u) {
      if (u == k) pk = pr[u];
      if (u == j) pj = pr[u];
    }
    g.C2[(m * N + k) * g.ldc + j] = pk * ((k == j ? 1.f : 0.f) - pj);
  }
  if (g.head_gprev) {
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      const int i = tid + c * kHeadThreads;
      if (i >= K) continue;
      float s = 0.f;
#pragma unroll
      for (int j = 0; j < kRowsMaxN; ++j) s += pr[j] * w[c][j];
#pragma unroll
      for (int k = 0; k < kRowsMaxN; ++k)
        if (k < N) g.head_gprev[(m * N + k) * K + i] = mask[c] * pr[k] * (w[c][k] - s);
    }
  }
}

}  // namespace

bool head_rows_applies(const GemmArgs &g) {
  return g.epilogue == EPI_HEAD && !g.bf16 && g.a_is_f32 && g.w_kn && g.S == 1 && !g.a_scale && !g.sub &&
         g.nbatch <= 1 && g.N >= 1 && g.N <= kRowsMaxN && g.K >= 1 && g.K <= 4 * kHeadThreads && g.M >= 1 &&
         g.M <= 2048 && g.C == nullptr;
}

hipError_t launch_head_rows(const GemmArgs &g, int mode, hipStream_t stream) {
  if (!head_rows_applies(g) || (mode != 0 && mode != 1)) return hipErrorInvalidValue;
  if (mode == 0 && (!g.labels || !g.C2)) return hipErrorInvalidValue;
  if (g.head_gprev && !g.head_mask) return hipErrorInvalidValue;
  const dim3 grid((unsigned)g.M), block(kHeadThreads);
  if (g.K <= kHeadThreads)
    PFG_KERNEL(head_rows_kernel<1>, grid, block, 0, stream, g, mode);
  else if (g.K <= 2 * kHeadThreads)
    PFG_KERNEL(head_rows_kernel<2>, grid, block, 0, stream, g, mode);
  else
    PFG_KERNEL(head_rows_kernel<4>, grid, block, 0, stream, g, mode);
  return hipGetLastError();
}

int head_split_shape(int64_t M, int64_t N, int64_t K) {
  if (N > 32 || K < 2048 || M > 1024) return 1;     // the fused head is the better one for these
  const int64_t row_tiles64 = (M + 63) / 64;
  // enough pieces for 128 tiles of 64 x 64 (what the tiled kernel wants), each a multiple of 64 long
  for (int Z = 2; Z <= 128; Z *= 2)
    if (Z * row_tiles64 >= 128) return (K % (64 * Z) == 0) ? Z : 1;
  return 1;
}

int head_split_pieces(const GemmArgs &g) {
  if (g.epilogue != EPI_HEAD || g.S != 1 || g.a_scale || g.sub || g.nbatch > 1 || !g.w_kn) return 1;
  return head_split_shape(g.M, g.N, g.K);
}

hipError_t launch_head_split(const GemmArgs &g, int Z, float *partials, hipStream_t stream) {
  if (Z < 2 || Z != head_split_pieces(g) || !partials || !g.labels || !g.C2) return hipErrorInvalidValue;
  const int Kz = g.K / Z;
  GemmArgs b = g;
  b.K = Kz;
  b.nbatch = Z;
  b.batch_A = Kz;                           // piece z: columns z Kz .. of A, rows z Kz .. of W [K, N]
  b.batch_W = (int64_t)Kz * g.ldw;
  b.batch_C = (int64_t)g.M * g.N;
  b.C = partials; b.ldc = g.N; b.C2 = nullptr;
  b.epilogue = EPI_NONE; b.bias = nullptr; b.labels = nullptr; b.loss = nullptr;
  b.head_gprev = nullptr; b.head_mask = nullptr; b.streaming = 0;
  hipError_t e = launch_gemm(b, stream);
  if (e != hipSuccess) return e;
  const int row_tiles = (g.M + 31) / 32;
  int groups = 1;
  if (g.head_gprev) {
    // the cotangent step of a row tile is shared out over workgroups of at least 32 columns each.
    // A thread walks the rows of its column one after the other, a load and a store per row, so
    // short walks matter more than few workgroups (adding the partial logits again is cheap):
    // up to four workgroups per compute unit
    const int cap = 1024 / row_tiles > 8 ? 1024 / row_tiles : 8;
    groups = g.K / 32;
    groups = groups < 1 ? 1 : (groups > cap ? cap : groups);
  }
  PFG_KERNEL(head_from_partials_kernel, dim3((unsigned)(row_tiles * groups)), dim3(kHeadThreads), 0, stream, g,
             partials, Z);
  return hipGetLastError();
}

}  // namespace pfg
