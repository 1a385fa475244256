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

}  // namespace

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
