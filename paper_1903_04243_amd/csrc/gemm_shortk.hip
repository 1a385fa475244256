// Matrix product with a SHORT contraction and very many rows: C[M, N] = A[M, K] W[K, N] (+ bias),
// K = 32, 64 or 128, float32.
//
// Section 3.4 folds the iteration index of matmul(X[i], W) into the rows of one product when W is
// loop-invariant; with every token of every sequence as a row (the input projection x W_x + b of the
// LSTM loops: 51 957 rows, K = 128, N = 1024) the product is long in M only.  On the LDS-tiled kernel
// a tile of such a product is four stages, all start-up: it never overlaps its loads with its MFMAs.
// Here the weight operand is what stays put: a workgroup stages a W tile of 128 columns in LDS once
// and its four waves stream row tiles of 32 rows past it, each wave on its own (no barrier after the
// staging): the A rows of a tile travel from global memory straight into the wave's registers (a lane
// = one row and half of the contraction, requested half a tile ahead of the products that use them),
// the W fragments come from LDS, and the 32 x 128 result leaves from the
// accumulators as 16-byte stores.  For that the 128 columns are dealt to the wave's four MFMA tiles
// in turn (column n0 + 4 l + e belongs to tile e, lane l), so that register r of the four tiles holds
// four neighbouring columns of one row.
//
// v_mfma_f32_32x32x2_f32: D[i][j] += A[i][k] B[k][j], lane (l32, half) supplies A[l32][half] and
// B[half][l32] and holds D[8 (r / 4) + 4 half + r % 4][l32] in register r.
#include <algorithm>

#include "common.h"

namespace pfg {

namespace {

constexpr int kThreads = 256;
constexpr int kColTile = 128;

// KG: groups of eight contraction steps (K = 8 KG)
template <int KG>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))
void gemm_shortk_kernel(const GemmArgs g, int col_tiles, int row_groups) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  float *ws = reinterpret_cast<float *>(smem_raw);       // [128 (tile e, lane l)][K + 4]
  constexpr int K = 8 * KG, WS = K + 4;
  const int tid = threadIdx.x, lane = tid & 63, half = lane >> 5, l32 = lane & 31;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  // The column tiles of a group of rows go to one XCD (workgroup ids are dealt to the eight XCDs in
  // turn), so that a row of A enters one L2 for all of them.
  const int xcd = blockIdx.x % 8, idx = blockIdx.x / 8;
  const int ct = idx % col_tiles, rg = (idx / col_tiles) * 8 + xcd;
  if (rg >= row_groups) return;
  const int n0 = ct * kColTile;
  const float *A = static_cast<const float *>(g.A);
  const float *W = static_cast<const float *>(g.W);

  // ---- the W tile, once: W[k][n0 + 4 c4 + e] -> ws[(32 e + c4)][k] ----
#pragma unroll
  for (int i = 0; i < KG; ++i) {
    const int k = (tid >> 5) + 8 * i, c4 = tid & 31;
    const f32x4 v = *reinterpret_cast<const f32x4 *>(W + (int64_t)k * g.ldw + n0 + 4 * c4);
#pragma unroll
    for (int e = 0; e < 4; ++e) ws[(32 * e + c4) * WS + k] = v[e];
  }
  f32x4 bias4 = {0.f, 0.f, 0.f, 0.f};
  if (g.epilogue == EPI_BIAS && g.bias) bias4 = *reinterpret_cast<const f32x4 *>(static_cast<const float *>(g.bias) + n0 + 4 * l32);
  __syncthreads();

  const int tiles_m = (g.M + 31) / 32;
  const int stride = row_groups * 4;
  int rt = rg * 4 + wv;
  if (rt >= tiles_m) return;
  // A lane's share of a row tile is K / 2 values = KG 16-byte pieces, fetched in two halves: the second
  // half of the current tile is requested before the products of its first half, the first half of
  // the next tile before the products of the second, so that every load has half a tile of MFMAs
  // (3 us at K = 128) to arrive and only one tile's worth of registers is held.
  constexpr int HG = KG / 2;
  auto request = [&](int tile, int part, f32x4 (&a)[HG]) {
    const int row = min(tile * 32 + l32, g.M - 1);            // rows past the end repeat the last one, never stored
    const float *src = A + (int64_t)row * g.a_batch_stride + 4 * half + 8 * HG * part;
#pragma unroll
    for (int gi = 0; gi < HG; ++gi) a[gi] = *reinterpret_cast<const f32x4 *>(src + 8 * gi);
  };
  const float *wrow = ws + l32 * WS + 4 * half;
  f32x16 acc[4];
  auto products = [&](const f32x4 (&a)[HG], int part) {
#pragma unroll
    for (int gi = 0; gi < HG; ++gi) {
      f32x4 wf[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) wf[e] = *reinterpret_cast<const f32x4 *>(wrow + 32 * e * WS + 8 * (gi + HG * part));
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          acc[e] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[gi][j], wf[e][j], acc[e], 0, 0, 0);
    }
  };
  f32x4 lo[HG], hi[HG];
  request(rt, 0, lo);
  auto tile = [&](int rt) {
    // the W fragments are the same for every tile: without this the compiler keeps all of them in
    // registers across the loop (256 of them at K = 128) and spills
    asm volatile("" ::: "memory");
    request(rt, 1, hi);
    __builtin_amdgcn_sched_barrier(0);       // the loads are issued here, not next to their use
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[e][r] = 0.f;
    products(lo, 0);
    request(min(rt + stride, tiles_m - 1), 0, lo);          // after the last tile: that tile once more, unused
    __builtin_amdgcn_sched_barrier(0);
    products(hi, 1);
    // A row past the end was computed from the last row's values and is stored onto the last row
    // (the same values again): no branch around the stores, so that the count of memory operations
    // in flight is known and a wait for the next tile's loads does not also wait for these stores.
    float *ccol = g.C + n0 + 4 * l32;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = min(rt * 32 + 4 * half + 8 * (r >> 2) + (r & 3), g.M - 1);
      const f32x4 v = f32x4{acc[0][r], acc[1][r], acc[2][r], acc[3][r]} + bias4;
      f32x4 *q = reinterpret_cast<f32x4 *>(ccol + (int64_t)row * g.ldc);
      if (g.streaming) __builtin_nontemporal_store(v, q);
      else *q = v;
    }
  };
  // The first tile apart from the loop: the loop is then entered with the same memory operations in
  // flight as it is re-entered with, and the waits inside it are counted for exactly that.
  tile(rt);
  for (rt += stride; rt < tiles_m; rt += stride) tile(rt);
}

template <int KG>
hipError_t launch_shortk(const GemmArgs &g, hipStream_t stream) {
  auto kern = gemm_shortk_kernel<KG>;
  constexpr int smem = kColTile * (8 * KG + 4) * 4;
  static bool attr_set = false;   // benign race: the attribute is idempotent
  if (!attr_set && smem > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int col_tiles = g.N / kColTile;
  const int tiles_m = (g.M + 31) / 32;
  // two workgroups per compute unit; then as few row groups as give every wave the same number of tiles
  int groups = std::max(1, 512 / col_tiles);
  const int per_wave = (tiles_m + 4 * groups - 1) / (4 * groups);
  groups = (tiles_m + 4 * per_wave - 1) / (4 * per_wave);
  const int64_t grid = (int64_t)((groups + 7) / 8) * 8 * col_tiles;
  PFG_KERNEL(kern, dim3((unsigned)grid), dim3(kThreads), smem, stream, g, col_tiles, groups);
  return hipGetLastError();
}

}  // namespace

bool gemm_shortk_applies(const GemmArgs &g) {
  if (g.bf16 || !g.a_is_f32 || !g.w_kn || g.a_scale || g.sub || g.a_km || g.conv_k > 0 || g.nbatch > 1 || g.sym_n > 0)
    return false;
  if (g.epilogue != EPI_NONE && g.epilogue != EPI_BIAS) return false;
  if (g.K != 32 && g.K != 64 && g.K != 128) return false;
  if (g.N < kColTile || g.N % kColTile) return false;
  // one row per iteration, at its own stride (a block shared by the iterations is not folded into rows here)
  if (g.S != 1 || g.a_batch_stride < g.K) return false;
  // enough rows for two workgroups on every compute unit to have several tiles each
  if (g.M < 16384 || (int64_t)g.M * g.N > 0x7fffffffffLL) return false;
  auto aligned = [](const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15) == 0; };
  if (!aligned(g.A) || !aligned(g.W) || !aligned(g.C) || !aligned(g.bias)) return false;
  return g.a_batch_stride % 4 == 0 && g.ldw % 4 == 0 && g.ldc % 4 == 0;
}

hipError_t launch_gemm_shortk(const GemmArgs &g, hipStream_t stream) {
  if (!gemm_shortk_applies(g)) return hipErrorInvalidValue;
  switch (g.K) {
    case 32: return launch_shortk<4>(g, stream);
    case 64: return launch_shortk<8>(g, stream);
    default: return launch_shortk<16>(g, stream);
  }
}

}  // namespace pfg
