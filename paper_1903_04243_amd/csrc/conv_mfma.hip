// Convolution blocks on the matrix cores WITHOUT a patch matrix, for feature maps small enough that
// an example's zero-padded image sits in LDS.
//
// Section 3.4's convolution rule folds the example index into the batch of output positions; the
// product over the rows (b, y, x) of a patch matrix is what the tiled kernel runs (gathering the
// patches while it stages them).  For a block with many input channels on a small map that staging,
// not the matrix pipe, sets the pace: every patch value is fetched k * k times.  Here a workgroup
// loads the padded image of its example once and the MFMA operands are read from it in place: the
// contraction index runs over (tap, channel), and for one tap the 32 positions of a tile are 32
// shifted addresses of the same LDS image.
//
//   conv_direct_kernel<NT, false>: forward product + bias, relu and 2 x 2 pooling of one example and
//       32 filters; pooled / which as relu_pool_kernel writes them, the pre-activation never leaves
//       the chip.
//   conv_direct_kernel<NT, true>:  cotangent of the block's input, din = dz convolved with the
//       filter flipped and transposed; replaces the patch-cotangent product and its gather.
//   conv_filter_direct_kernel<TT>: the per-example filter gradient (both operands stacked over the
//       examples, Section 3.4): for each tap, in_shifted^T dz over the positions.
//   conv_filter_rows_kernel<MT>:   the same gradient for a block with few input channels (a first
//       layer): the rows (tap, channel) fill one or two MFMA tiles, each lane reading its own shifted
//       image value.
// The host side takes each of them only from the batch size on where it was measured faster than the
// tiled products (a workgroup here costs the same however few examples there are).
//
// v_mfma_f32_32x32x2_f32 computes D[i][j] += A[i][k] B[k][j] with lane (l32, half) supplying
// A[l32][half] and B[half][l32], and holding D[8 (r / 4) + 4 half + r % 4][l32] in register r.
#include <algorithm>

#include "common.h"

namespace pfg {

namespace {

constexpr int kThreads = 256;      // four waves, one per SIMD
constexpr int kStageMax = 12;      // 16-byte pieces of a filter chunk a thread carries in registers

// n / d for 0 <= n < 2^24 and d >= 1 with the reciprocal given: the float product is off by one at
// most, which the remainder shows (a 32-bit division by a run-time divisor costs ten times as much)
__device__ __forceinline__ int div_small(int n, int d, float inv) {
  int q = (int)((float)n * inv);
  const int r = n - q * d;
  if (r < 0) --q;
  if (r >= d) ++q;
  return q;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// The sum of `v` over the four waves of a workgroup in the order of the waves, through `slot` (four
// floats of LDS nobody else touches meanwhile); valid in thread 0.
__device__ __forceinline__ float workgroup_sum(float v, float *slot, int wv, int lane) {
  v = wave_sum(v);
  if (lane == 0) slot[wv] = v;
  __syncthreads();
  return ((slot[0] + slot[1]) + slot[2]) + slot[3];
}

constexpr int kCopyBatch = 16;     // 16-byte loads a thread has in flight while an image is copied to LDS

// Copies the zero-padded band of an image to LDS: rows row0 - p .. of `nrows` padded rows, PW padded
// columns, c4 16-byte pieces per position (the image has `stride` floats per position, the LDS copy
// `lds_stride`).  The loads of a batch are issued together, without branches between them: one
// memory latency per batch, not per piece.
__device__ __forceinline__ void copy_padded_band(const float *src, int h, int w, int stride, int c4, int row0,
                                                 int p, int nrows, int PW, float *dst, int lds_stride, int tid,
                                                 int threads) {
  const int total = nrows * PW * c4;
  const float inv_c4 = 1.f / (float)c4, inv_pw = 1.f / (float)PW;
  for (int e0 = 0; e0 < total; e0 += kCopyBatch * threads) {
    f32x4 v[kCopyBatch];
    int at[kCopyBatch];
#pragma unroll
    for (int u = 0; u < kCopyBatch; ++u) {
      const int e = e0 + u * threads + tid;
      const int ec = min(e, total - 1);
      const int cell = div_small(ec, c4, inv_c4), qq = ec - cell * c4;
      const int r = div_small(cell, PW, inv_pw), cx = cell - r * PW;
      const int y = row0 + r - p, x = cx - p;
      const bool inside = y >= 0 && y < h && x >= 0 && x < w;
      const float *q = inside ? src + (y * w + x) * stride + 4 * qq : src;
      v[u] = *reinterpret_cast<const f32x4 *>(q);
      if (!inside) v[u] = f32x4{0.f, 0.f, 0.f, 0.f};
      at[u] = e < total ? cell * lds_stride + 4 * qq : -1;
    }
#pragma unroll
    for (int u = 0; u < kCopyBatch; ++u)
      if (at[u] >= 0) *reinterpret_cast<f32x4 *>(dst + at[u]) = v[u];
  }
}

struct ConvDirectArgs {
  const float *in;       // [B, h, w, q]: the image whose windows are read (forward: the block's input, reverse: dz)
  const float *Wc;       // [k, k, ci, co]
  const float *bias;     // forward: [co] or null
  float *out;            // forward: pooled [B, h / 2, w / 2, co]; reverse: din [B, h, w, ci]
  uint8_t *which;        // forward: [B, h / 2, w / 2, co]
  int h, w, k, ci, co;
  int q;                 // channels of `in` = length of the contraction per tap (forward ci, reverse co)
  int o_total;           // channels of the output (forward co, reverse ci), a multiple of 32
  int tiles;             // tiles of 32 positions in an example, ceil(h w / 32)
  int splits;            // workgroups an example's tiles are dealt to (forward: 1)
  int tc;                // taps per filter chunk
  int rows_max;          // rows of the padded image a workgroup keeps (the most over the splits)
};

// out[pos, o] = sum over taps (dy, dx) and channels c of  img[pos + (dy, dx), c] F[(dy, dx), c, o]
// for the positions of NT tiles at most and 32 output channels.  REVERSE = false: F = Wc as stored.
// REVERSE = true: F[(dy, dx), n, c] = Wc[(k - 1 - dy, k - 1 - dx), c, n], transposed while it is staged.
// The four waves split the contraction (wave v takes the channel octets v, v + 4, ... of every tap)
// and each keeps all NT tiles, so a filter fragment serves NT products; the partial sums meet in
// LDS and are added in the order of the waves.  The filter passes through LDS in chunks of tc taps,
// the next chunk travelling in registers while the current one is used.
template <int NT, bool REVERSE>
__global__ __launch_bounds__(kThreads) void conv_direct_kernel(const ConvDirectArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  float *smem = reinterpret_cast<float *>(smem_raw);
  constexpr int FS = REVERSE ? 33 : 32;      // row stride of the staged filter (33: written transposed)
  const int tid = threadIdx.x, lane = tid & 63, half = lane >> 5, l32 = lane & 31;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);      // the same in every lane: keeps the loops over it scalar
  const int k = a.k, p = (k - 1) / 2, h = a.h, w = a.w, hw = h * w, PW = w + k - 1;
  const int Q = a.q, IS = Q + 4, taps = k * k, octs = Q / 8, Q4 = Q / 4;

  int idx = blockIdx.x;
  const int split = idx % a.splits;
  idx /= a.splits;
  const int otiles = a.o_total / 32;
  const int o0 = (idx % otiles) * 32;
  const int64_t b = idx / otiles;
  const int t_lo = split * NT, nt = min(NT, a.tiles - t_lo);
  const int pos_lo = t_lo * 32, pos_hi = min(pos_lo + nt * 32, hw);
  const int y_lo = pos_lo / w, y_hi = (pos_hi - 1) / w;
  const int nrows = y_hi - y_lo + k;         // padded rows y_lo .. y_hi + k - 1 hold every window of these positions

  float *img = smem;                                   // [nrows][PW][IS], IS = Q + 4: conflict-free 16-byte reads
  float *flt = smem + a.rows_max * PW * IS;            // [tc Q][FS]

  // ---- staging plan of a filter chunk: piece i of this thread, relative to the chunk's first tap ----
  // forward: piece = (row, 4 outputs), row = (tap in chunk) Q + channel, copied as it lies;
  // reverse: piece = (tap in chunk, output channel, 4 contraction channels), written transposed.
  int64_t g_off[kStageMax];
  int l_off[kStageMax];
  const int chunk_pieces = a.tc * Q * 8;
  const float inv_q4 = 1.f / (float)Q4;
#pragma unroll
  for (int i = 0; i < kStageMax; ++i) {
    const int e = tid + i * kThreads;
    if (REVERSE) {
      const int eq = div_small(e, Q4, inv_q4);           // = tl * 32 + oc
      const int nq = e - eq * Q4, oc = eq & 31, tl = eq >> 5;
      // data tap t reads the filter's tap taps - 1 - t
      g_off[i] = ((int64_t)(taps - 1 - tl) * a.ci + o0 + oc) * a.co + 4 * nq;
      l_off[i] = (tl * Q + 4 * nq) * FS + oc;
    } else {
      const int c4 = e % 8, row = e / 8;
      g_off[i] = (int64_t)row * a.co + o0 + 4 * c4;
      l_off[i] = row * FS + 4 * c4;
    }
  }
  const int64_t chunk_step = REVERSE ? -(int64_t)a.tc * a.ci * a.co : (int64_t)a.tc * Q * a.co;
  f32x4 stage[kStageMax];
  auto fetch_chunk = [&](int c) {
    const int live = min(a.tc, taps - c * a.tc) * Q * 8;
    const float *src = a.Wc + c * chunk_step;
#pragma unroll
    for (int i = 0; i < kStageMax; ++i)
      if (i * kThreads < chunk_pieces && tid + i * kThreads < live)
        stage[i] = *reinterpret_cast<const f32x4 *>(src + g_off[i]);
  };
  auto store_chunk = [&](int c) {
    const int live = min(a.tc, taps - c * a.tc) * Q * 8;
#pragma unroll
    for (int i = 0; i < kStageMax; ++i)
      if (i * kThreads < chunk_pieces && tid + i * kThreads < live) {
        if (REVERSE) {
#pragma unroll
          for (int j = 0; j < 4; ++j) flt[l_off[i] + j * FS] = stage[i][j];
        } else {
          *reinterpret_cast<f32x4 *>(flt + l_off[i]) = stage[i];
        }
      }
  };

  fetch_chunk(0);

  // ---- the band of the padded image ----
  copy_padded_band(a.in + b * hw * Q, h, w, Q, Q4, y_lo, p, nrows, PW, img, IS, tid, kThreads);
  store_chunk(0);

  // window origin of this lane's position in every tile (lanes past the last position repeat it; a
  // tile past the workgroup's last one repeats the first: computed like the others, never stored)
  int off[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int pos = min(pos_lo + (t < nt ? t : 0) * 32 + l32, pos_hi - 1);
    const int y = div_small(pos, w, 1.f / (float)w), x = pos - y * w;
    off[t] = ((y - y_lo) * PW + x) * IS + 4 * half;
  }
  f32x16 acc[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
  __syncthreads();

  // A group = one tap and eight channels = four MFMA steps on every tile.  This wave's groups of a
  // chunk are g = wv, wv + 4, ...; (tl, oc8) = (g / octs, g % octs) and the tap's (dy, dx) are
  // carried along.  The operands of the next group are requested before the products of this one.
  struct Cursor { int tl, oc8, dy, dx; };
  auto advance = [&](Cursor &q) {
    q.oc8 += 4;
    while (q.oc8 >= octs) {
      q.oc8 -= octs;
      ++q.tl;
      if (++q.dx == k) { q.dx = 0; ++q.dy; }
    }
  };
  auto request = [&](const Cursor &q, float (&fa)[4], f32x4 (&xb)[NT]) {
    const float *frow = flt + (q.tl * Q + q.oc8 * 8 + 4 * half) * FS + l32;
#pragma unroll
    for (int j = 0; j < 4; ++j) fa[j] = frow[j * FS];
    const float *xrow = img + (q.dy * PW + q.dx) * IS + q.oc8 * 8;
#pragma unroll
    for (int t = 0; t < NT; ++t) xb[t] = *reinterpret_cast<const f32x4 *>(xrow + off[t]);
  };
  auto products = [&](const float (&fa)[4], const f32x4 (&xb)[NT]) {
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[j], xb[t][j], acc[t], 0, 0, 0);
  };

  const int nchunks = (taps + a.tc - 1) / a.tc;
  for (int c = 0; c < nchunks; ++c) {
    if (c + 1 < nchunks) fetch_chunk(c + 1);
    const int tcn = min(a.tc, taps - c * a.tc);
    Cursor q{0, wv - 4, (c * a.tc) / k, (c * a.tc) % k};
    advance(q);
    float fa0[4], fa1[4];
    f32x4 xb0[NT], xb1[NT];
    if (q.tl < tcn) request(q, fa0, xb0);
    while (q.tl < tcn) {
      advance(q);
      if (q.tl < tcn) request(q, fa1, xb1);
      products(fa0, xb0);
      if (q.tl >= tcn) break;
      advance(q);
      if (q.tl < tcn) request(q, fa0, xb0);
      products(fa1, xb1);
    }
    __syncthreads();
    if (c + 1 < nchunks) {
      store_chunk(c + 1);
      __syncthreads();
    }
  }

  // ---- the four partial sums meet in LDS: part[wave][position][36], a lane's four consecutive
  // output channels of a position as one 16-byte piece; added in the order of the waves ----
  float *part = smem;
  const int wstride = nt * 32 * 36;
  const int n4 = tid & 7;                    // the four channels this thread finishes (kThreads % 8 == 0)
  f32x4 bv = {0.f, 0.f, 0.f, 0.f};
  if (!REVERSE && a.bias) bv = *reinterpret_cast<const f32x4 *>(a.bias + o0 + 4 * n4);
#pragma unroll
  for (int t = 0; t < NT; ++t)
    if (t < nt) {
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const f32x4 v = {acc[t][4 * q4], acc[t][4 * q4 + 1], acc[t][4 * q4 + 2], acc[t][4 * q4 + 3]};
        *reinterpret_cast<f32x4 *>(part + wv * wstride + (t * 32 + l32) * 36 + 8 * q4 + 4 * half) = v;
      }
    }
  __syncthreads();
  auto total_at = [&](int pl) {
    const float *q = part + pl * 36 + 4 * n4;
    f32x4 sum = *reinterpret_cast<const f32x4 *>(q);
    sum += *reinterpret_cast<const f32x4 *>(q + wstride);
    sum += *reinterpret_cast<const f32x4 *>(q + 2 * wstride);
    sum += *reinterpret_cast<const f32x4 *>(q + 3 * wstride);
    return sum;
  };
  const int npos = pos_hi - pos_lo;

  if (REVERSE) {
    // din[b, pos, o0 + n]: a thread takes four channels of a position
    float *dst = a.out + (b * hw + pos_lo) * a.o_total + o0 + 4 * n4;
    for (int pl = tid >> 3; pl < npos; pl += kThreads / 8)
      *reinterpret_cast<f32x4 *>(dst + (int64_t)pl * a.o_total) = total_at(pl);
  } else {
    // relu and 2 x 2 pooling exactly as relu_pool_kernel takes them: the first maximum in the order
    // (0,0), (0,1), (1,0), (1,1) of the window; a thread takes four channels of a pooled cell
    const int ho = h / 2, wo = w / 2;
    const float inv_wo = 1.f / (float)wo;
    for (int cell = tid >> 3; cell < ho * wo; cell += kThreads / 8) {
      const int yo = div_small(cell, wo, inv_wo), xo = cell - yo * wo;
      f32x4 best = {-1.f, -1.f, -1.f, -1.f};
      uint32_t arg = 0;
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        const f32x4 z = total_at((2 * yo + (d >> 1)) * w + 2 * xo + (d & 1)) + bv;
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
          const float r = z[qd] > 0.f ? z[qd] : 0.f;
          if (r > best[qd]) {
            best[qd] = r;
            arg = (arg & ~(0xffu << (8 * qd))) | ((uint32_t)d << (8 * qd));
          }
        }
      }
      const int64_t at = ((b * ho + yo) * wo + xo) * a.co + o0 + 4 * n4;
      *reinterpret_cast<f32x4 *>(a.out + at) = best;
      *reinterpret_cast<uint32_t *>(a.which + at) = arg;
    }
  }
}

struct ConvFilterArgs {
  const float *in;     // [B, h, w, ci]
  const float *dz;     // [B, h, w, co]
  float *dWc;          // [B, k k ci, co]
  int h, w, k, ci, co;
  int streaming;       // non-temporal stores (the gradients are not read back)
  float *sq_part;      // set: no gradient is stored, only the sum of its squares per workgroup, [B, workgroups per example]
};

// dWc[b, (dy, dx, c), n] = sum over the positions of in[b, pos + (dy, dx) - p, c] dz[b, pos, n] for 32
// channels c and 32 filters n of one example.  The padded image (its 32 channels) and the dz columns
// sit in LDS; a wave takes up to TT taps and walks the positions once for all of them, so a dz
// fragment serves TT products.  Stores go through LDS to leave as 16-byte pieces.
template <int TT>
__global__ __launch_bounds__(kThreads) void conv_filter_direct_kernel(const ConvFilterArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  float *smem = reinterpret_cast<float *>(smem_raw);
  const int tid = threadIdx.x, lane = tid & 63, half = lane >> 5, l32 = lane & 31;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);      // the same in every lane: keeps the loops over it scalar
  const int k = a.k, p = (k - 1) / 2, h = a.h, w = a.w, hw = h * w, PW = w + k - 1, PH = h + k - 1;
  const int taps = k * k;
  int idx = blockIdx.x;
  const int ntiles = a.co / 32, ctiles = a.ci / 32;
  const int n0 = (idx % ntiles) * 32;
  idx /= ntiles;
  const int c0 = (idx % ctiles) * 32;
  const int64_t b = idx / ctiles;

  float *img = smem;                        // [PH][PW][32]
  float *dzs = smem + PH * PW * 32;         // [hw][32]
  {
    // the dz columns: the first batch of loads travels while the image is copied
    const float *dsrc = a.dz + b * hw * a.co + n0;
    const int total = hw * 8;
    for (int e0 = 0; e0 < total; e0 += kCopyBatch * kThreads) {
      f32x4 v[kCopyBatch];
#pragma unroll
      for (int u = 0; u < kCopyBatch; ++u) {
        const int e = min(e0 + u * kThreads + tid, total - 1);
        v[u] = *reinterpret_cast<const f32x4 *>(dsrc + (int64_t)(e >> 3) * a.co + 4 * (e & 7));
      }
      if (e0 == 0) copy_padded_band(a.in + b * hw * a.ci + c0, h, w, a.ci, 8, 0, p, PH, PW, img, 32, tid, kThreads);
#pragma unroll
      for (int u = 0; u < kCopyBatch; ++u) {
        const int e = e0 + u * kThreads + tid;
        if (e < total) *reinterpret_cast<f32x4 *>(dzs + (e >> 3) * 32 + 4 * (e & 7)) = v[u];
      }
    }
  }
  // this wave's taps: contiguous runs, the first waves one longer when they do not divide
  const int base = taps / 4, extra = taps % 4;
  const int my = base + (wv < extra ? 1 : 0);
  const int tap0 = wv * base + min(wv, extra);
  int toff[TT];
#pragma unroll
  for (int tt = 0; tt < TT; ++tt) {
    const int tap = tap0 + min(tt, my - 1);
    const int dy = tap / k, dx = tap - dy * k;
    toff[tt] = (dy * PW + dx) * 32;
  }
  f32x16 acc[TT];
#pragma unroll
  for (int tt = 0; tt < TT; ++tt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[tt][r] = 0.f;
  __syncthreads();

  // Positions two at a time (one per half-wave); w is even, so a pair never straddles a row and
  // h w / 2 is even.  A wave with fewer than TT taps repeats its last one (computed, never stored).
  // The operands of the next step are requested before the products of this one.
  {
    const float *ap = img + half * 32 + l32, *bp = dzs + half * 32 + l32;
    int xi = 0;                      // pairs done in the current row
    const int wrap = (PW - w) * 32, pairs = w / 2, steps = hw / 2;
    auto request = [&](float (&av)[TT], float &bv) {
      bv = *bp;
#pragma unroll
      for (int tt = 0; tt < TT; ++tt) av[tt] = ap[toff[tt]];
    };
    auto advance = [&]() {
      ap += 64;
      bp += 64;
      if (++xi == pairs) { xi = 0; ap += wrap; }
    };
    auto products = [&](const float (&av)[TT], float bv) {
#pragma unroll
      for (int tt = 0; tt < TT; ++tt) acc[tt] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv, av[tt], acc[tt], 0, 0, 0);
    };
    float av0[TT], av1[TT], bv0, bv1;
    request(av0, bv0);
    for (int st = 0; st < steps; st += 2) {
      advance();
      request(av1, bv1);
      products(av0, bv0);
      if (st + 2 < steps) advance();       // past the end: the last step's operands once more, unused
      request(av0, bv0);
      products(av1, bv1);
    }
  }
  __syncthreads();

  // A tap's tile comes out of the product as [filter][channel] (D rows = filters), so a lane holds four
  // consecutive filters of its channel per register quad: written to this wave's LDS slab
  // [32 channels][36] as 16-byte pieces and read back row by row for 16-byte stores.  The slab is the
  // wave's own: its LDS operations execute in order, no workgroup barrier is needed between the taps.
  if (a.sq_part) {
    // only the norm is wanted: this workgroup's share of the sum of squares (dead taps left out)
    float sq = 0.f;
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
      if (tt < my)
#pragma unroll
        for (int r = 0; r < 16; ++r) sq += acc[tt][r] * acc[tt][r];
    sq = workgroup_sum(sq, smem, wv, lane);
    if (tid == 0) a.sq_part[blockIdx.x] = sq;
    return;
  }
  float *slab = smem + wv * (32 * 36);
  float *dst = a.dWc + b * (int64_t)taps * a.ci * a.co;
#pragma unroll
  for (int tt = 0; tt < TT; ++tt) {
    if (tt < my) {
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const f32x4 v = {acc[tt][4 * q4], acc[tt][4 * q4 + 1], acc[tt][4 * q4 + 2], acc[tt][4 * q4 + 3]};
        *reinterpret_cast<f32x4 *>(slab + l32 * 36 + 8 * q4 + 4 * half) = v;
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
      const int tap = tap0 + tt;
#pragma unroll
      for (int ps = 0; ps < 4; ++ps) {
        const int row = ps * 8 + (lane >> 3), c4 = lane & 7;
        const f32x4 v = *reinterpret_cast<const f32x4 *>(slab + row * 36 + 4 * c4);
        f32x4 *q = reinterpret_cast<f32x4 *>(dst + ((int64_t)tap * a.ci + c0 + row) * a.co + n0 + 4 * c4);
        if (a.streaming) __builtin_nontemporal_store(v, q);
        else *q = v;
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
  }
}

// The same gradient for a block with FEW input channels (a first layer: k k c_in <= 32 MT): the rows
// (tap, channel) of the gradient fill one or two MFMA tiles, a lane owning one row and reading its
// shifted image value through its own offset; the four waves split the positions and their partial
// tiles meet in LDS.  A workgroup = one example and 32 filters; the padded image (all channels) and
// the dz columns sit in LDS.  Image rows are padded to an odd number of floats, so that the taps of
// a column of the filter fall into different banks.
template <int MT>
__global__ __launch_bounds__(kThreads) void conv_filter_rows_kernel(const ConvFilterArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  float *smem = reinterpret_cast<float *>(smem_raw);
  const int tid = threadIdx.x, lane = tid & 63, half = lane >> 5, l32 = lane & 31;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int k = a.k, p = (k - 1) / 2, h = a.h, w = a.w, hw = h * w, PW = w + k - 1, PH = h + k - 1;
  const int ci = a.ci, M = k * k * ci;
  const int RS = (PW * ci) | 1;               // floats per padded image row
  const int ntiles = a.co / 32;
  const int n0 = (blockIdx.x % ntiles) * 32;
  const int64_t b = blockIdx.x / ntiles;

  float *img = smem;                           // [PH][RS]
  float *dzs = smem + ((PH * RS + 3) & ~3);    // [hw][32]
  {
    // the dz columns: the first batch of loads travels while the image is copied
    const float *dsrc = a.dz + b * hw * a.co + n0;
    const int total = hw * 8;
    for (int e0 = 0; e0 < total; e0 += kCopyBatch * kThreads) {
      f32x4 v[kCopyBatch];
#pragma unroll
      for (int u = 0; u < kCopyBatch; ++u) {
        const int e = min(e0 + u * kThreads + tid, total - 1);
        v[u] = *reinterpret_cast<const f32x4 *>(dsrc + (int64_t)(e >> 3) * a.co + 4 * (e & 7));
      }
      if (e0 == 0) {
        // the image, value by value (rows of w c_in floats land at odd strides), a batch of loads at a time
        const float *src = a.in + b * hw * ci;
        const int wc = w * ci, row_floats = PW * ci, all = PH * row_floats;
        const float inv_row = 1.f / (float)row_floats;
        for (int i0 = 0; i0 < all; i0 += 8 * kThreads) {
          float x[8];
          int at[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const int i = i0 + u * kThreads + tid, ic = min(i, all - 1);
            const int r = div_small(ic, row_floats, inv_row), rem = ic - r * row_floats;
            const int y = r - p, xc = rem - p * ci;
            const bool inside = y >= 0 && y < h && xc >= 0 && xc < wc;
            x[u] = src[inside ? y * wc + xc : 0];
            if (!inside) x[u] = 0.f;
            at[u] = i < all ? r * RS + rem : -1;
          }
#pragma unroll
          for (int u = 0; u < 8; ++u)
            if (at[u] >= 0) img[at[u]] = x[u];
        }
      }
#pragma unroll
      for (int u = 0; u < kCopyBatch; ++u) {
        const int e = e0 + u * kThreads + tid;
        if (e < total) *reinterpret_cast<f32x4 *>(dzs + (e >> 3) * 32 + 4 * (e & 7)) = v[u];
      }
    }
  }
  // this lane's row (tap, channel) in every tile: where its value sits relative to the window origin
  int roff[MT];
  const float inv_ci = 1.f / (float)ci, inv_k = 1.f / (float)k;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int m = min(mt * 32 + l32, M - 1);
    const int tap = div_small(m, ci, inv_ci), c = m - tap * ci;
    const int dy = div_small(tap, k, inv_k), dx = tap - dy * k;
    roff[mt] = dy * RS + dx * ci + c;
  }
  // two accumulators per tile, taken in turn: consecutive products do not wait for each other
  f32x16 acc[MT], acc2[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[mt][r] = acc2[mt][r] = 0.f;
  __syncthreads();

  // Positions two at a time (one per half-wave; w is even, a pair never straddles a row); this wave's
  // share of the pairs is a contiguous run.  D rows = filters, D columns = gradient rows.  A product
  // is short against the latency of its LDS reads, so the operands of four pairs are requested
  // together, one such group ahead of the products; past the end of the run the last pair is read
  // again with its dz values replaced by zero.
  {
    const int steps = hw / 2, pairs = w / 2;
    const int s_lo = (wv * steps) / 4, s_hi = ((wv + 1) * steps) / 4;
    const int y0 = div_small(s_lo, pairs, 1.f / (float)pairs);
    int xi = s_lo - y0 * pairs, st = s_lo;
    const float *ap = img + y0 * RS + (2 * xi + half) * ci;
    const float *bp = dzs + (2 * s_lo + half) * 32 + l32;
    const int wrap = RS - w * ci;
    auto request4 = [&](float (&av)[4][MT], float (&bv)[4]) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        bv[u] = *bp;
        if (st >= s_hi) bv[u] = 0.f;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) av[u][mt] = ap[roff[mt]];
        if (st + 1 < s_hi) {
          ap += 2 * ci;
          bp += 64;
          if (++xi == pairs) { xi = 0; ap += wrap; }
        }
        ++st;
      }
    };
    auto products4 = [&](const float (&av)[4][MT], const float (&bv)[4]) {
#pragma unroll
      for (int u = 0; u < 4; u += 2)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          acc[mt] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv[u], av[u][mt], acc[mt], 0, 0, 0);
          acc2[mt] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv[u + 1], av[u + 1][mt], acc2[mt], 0, 0, 0);
        }
    };
    if (s_lo < s_hi) {
      float av0[4][MT], av1[4][MT], bv0[4], bv1[4];
      request4(av0, bv0);
      for (int done = s_lo; done < s_hi; done += 8) {
        request4(av1, bv1);
        products4(av0, bv0);
        request4(av0, bv0);
        products4(av1, bv1);
      }
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mt][r] += acc2[mt][r];
  }
  __syncthreads();

  // the four partial tiles meet in LDS as 16-byte pieces part[wave][tile][row][36], added in the
  // order of the waves; a thread finishes four filters of a gradient row
  float *part = smem;
  const int wstride = MT * 32 * 36;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const f32x4 v = {acc[mt][4 * q4], acc[mt][4 * q4 + 1], acc[mt][4 * q4 + 2], acc[mt][4 * q4 + 3]};
      *reinterpret_cast<f32x4 *>(part + wv * wstride + (mt * 32 + l32) * 36 + 8 * q4 + 4 * half) = v;
    }
  __syncthreads();
  float *dst = a.dWc + b * (int64_t)M * a.co + n0;
  float sq = 0.f;
  for (int e = tid; e < M * 8; e += kThreads) {
    const int n4 = e & 7, m = e >> 3;
    const float *q = part + m * 36 + 4 * n4;
    f32x4 sum = *reinterpret_cast<const f32x4 *>(q);
    sum += *reinterpret_cast<const f32x4 *>(q + wstride);
    sum += *reinterpret_cast<const f32x4 *>(q + 2 * wstride);
    sum += *reinterpret_cast<const f32x4 *>(q + 3 * wstride);
    if (a.sq_part) {
      sq += (sum[0] * sum[0] + sum[1] * sum[1]) + (sum[2] * sum[2] + sum[3] * sum[3]);
      continue;
    }
    f32x4 *out = reinterpret_cast<f32x4 *>(dst + (int64_t)m * a.co + 4 * n4);
    if (a.streaming) __builtin_nontemporal_store(sum, out);
    else *out = sum;
  }
  if (a.sq_part) {
    // only the norm is wanted: the sum of squares of this workgroup's 32 filters
    __syncthreads();                         // part[] has been read: its first floats serve as the slot
    sq = workgroup_sum(sq, smem, wv, lane);
    if (tid == 0) a.sq_part[blockIdx.x] = sq;
  }
}

int lds_limit() {
  static int limit = -1;
  if (limit < 0) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess)
      v = 0;
    limit = v;
  }
  return limit;
}

bool aligned16(const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15) == 0; }

// Geometry of a direct launch: tiles per workgroup (1 .. 8), splits, taps per chunk, LDS bytes.
struct DirectShape {
  int nt, splits, tc, rows_max;
  size_t smem;
  bool ok;
};

DirectShape direct_shape(int64_t B, int h, int w, int k, int q, int o_total, bool reverse) {
  DirectShape s{};
  if (B < 1 || h < 2 || w < 2 || k < 1 || k % 2 == 0 || q < 8 || q % 8 || o_total < 32 || o_total % 32) return s;
  const int hw = h * w, tiles = (hw + 31) / 32, PW = w + k - 1, IS = q + 4, taps = k * k;
  const int64_t per_example = o_total / 32;
  int nt = 0;
  if (!reverse) {
    // pooling windows must not be cut: one workgroup keeps all tiles of its example
    if (tiles > 8) return s;
    nt = tiles;
  } else {
    // Workgroups per example: a workgroup costs about 20 us whatever it does (launch, image band,
    // first filter chunk, epilogue) plus 6 us per tile, and one workgroup fits a compute unit, so the
    // launch runs in rounds of 256; the split with the cheapest estimate wins (measured at 14 x 14 x
    // 64 -> 32, 5 x 5: one tile 25 us, four 45 us, seven 58 us; 288 workgroups of three tiles 68 us)
    double best = 1e30;
    for (int sp = (tiles + 7) / 8; sp <= tiles; ++sp) {
      const int per = (tiles + sp - 1) / sp;
      const int64_t wgs = B * per_example * ((tiles + per - 1) / per);
      const double cost = (double)((wgs + 255) / 256) * (20.0 + 6.0 * per);
      if (cost < best) { best = cost; nt = per; }
    }
  }
  s.nt = nt;
  s.splits = (tiles + nt - 1) / nt;
  for (int sp = 0; sp < s.splits; ++sp) {
    const int pos_lo = sp * nt * 32, pos_hi = std::min(pos_lo + nt * 32, hw);
    s.rows_max = std::max(s.rows_max, (pos_hi - 1) / w - pos_lo / w + k);
  }
  const int fs = reverse ? 33 : 32;
  const int tc_regs = 32 * kStageMax / q;     // tc q 8 pieces over 256 threads, kStageMax each
  if (tc_regs < 1) return s;
  const size_t img_bytes = (size_t)s.rows_max * PW * IS * 4;
  const int nt_live = std::min(nt, tiles);
  const size_t red_bytes = (size_t)4 * nt_live * 32 * 36 * 4;
  const int limit = lds_limit();
  int tc = std::min(taps, tc_regs);
  while (tc > 1 && img_bytes + (size_t)tc * q * fs * 4 > (size_t)limit) --tc;
  // chunks of equal length where that costs no extra chunk
  const int nchunks = (taps + tc - 1) / tc;
  tc = (taps + nchunks - 1) / nchunks;
  s.tc = tc;
  s.smem = std::max(img_bytes + (size_t)tc * q * fs * 4, red_bytes);
  s.ok = s.smem <= (size_t)limit && B * per_example * s.splits <= 0x7fffffffLL;
  return s;
}

template <int NT, bool REVERSE>
hipError_t launch_direct(const ConvDirectArgs &a, int64_t wgs, size_t smem, hipStream_t stream) {
  auto kern = conv_direct_kernel<NT, REVERSE>;
  static bool attr_set = false;   // benign race: the attribute is idempotent
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds_limit());
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  PFG_KERNEL(kern, dim3((unsigned)wgs), dim3(kThreads), smem, stream, a);
  return hipGetLastError();
}

template <bool REVERSE>
hipError_t launch_direct_nt(const ConvDirectArgs &a, int nt, int64_t wgs, size_t smem, hipStream_t stream) {
  switch (nt) {
    case 1: return launch_direct<1, REVERSE>(a, wgs, smem, stream);
    case 2: return launch_direct<2, REVERSE>(a, wgs, smem, stream);
    case 3: return launch_direct<3, REVERSE>(a, wgs, smem, stream);
    case 4: return launch_direct<4, REVERSE>(a, wgs, smem, stream);
    case 5: return launch_direct<5, REVERSE>(a, wgs, smem, stream);
    case 6: return launch_direct<6, REVERSE>(a, wgs, smem, stream);
    case 7: return launch_direct<7, REVERSE>(a, wgs, smem, stream);
    case 8: return launch_direct<8, REVERSE>(a, wgs, smem, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

bool conv_direct_forward_applies(const float *in, const float *Wc, const float *bias, int64_t B, int32_t h,
                                 int32_t w, int32_t ci, int32_t k, int32_t co, const float *pooled,
                                 const uint8_t *which) {
  if (!in || !Wc || !pooled || !which || h % 2 || w % 2) return false;
  if (!aligned16(in) || !aligned16(Wc) || !aligned16(bias) || !aligned16(pooled) ||
      (reinterpret_cast<uintptr_t>(which) & 3))
    return false;
  // below 64 taps per output the plain-ALU kernel of the first layers is the faster one
  if ((int64_t)k * k * ci < 64) return false;
  // a workgroup takes a whole example however few there are (32 us at 14 x 14 x 32, 5 x 5); below
  // half a chip of workgroups the tiled product over the gathered patches is faster (B = 32: 20 us)
  if (B * (co / 32) < 128) return false;
  return direct_shape(B, h, w, k, ci, co, false).ok;
}

hipError_t launch_conv_direct_forward(const float *in, const float *Wc, const float *bias, int64_t B, int32_t h,
                                      int32_t w, int32_t ci, int32_t k, int32_t co, float *pooled,
                                      uint8_t *which, hipStream_t stream) {
  if (!conv_direct_forward_applies(in, Wc, bias, B, h, w, ci, k, co, pooled, which)) return hipErrorInvalidValue;
  const DirectShape s = direct_shape(B, h, w, k, ci, co, false);
  ConvDirectArgs a{};
  a.in = in; a.Wc = Wc; a.bias = bias; a.out = pooled; a.which = which;
  a.h = h; a.w = w; a.k = k; a.ci = ci; a.co = co; a.q = ci; a.o_total = co;
  a.tiles = (h * w + 31) / 32; a.splits = s.splits; a.tc = s.tc; a.rows_max = s.rows_max;
  return launch_direct_nt<false>(a, s.nt, B * (co / 32) * s.splits, s.smem, stream);
}

bool conv_direct_reverse_applies(const float *dz, const float *Wc, int64_t B, int32_t h, int32_t w, int32_t ci,
                                 int32_t k, int32_t co, const float *din) {
  if (!dz || !Wc || !din) return false;
  if (!aligned16(dz) || !aligned16(Wc) || !aligned16(din)) return false;
  if (co % 4 || ci % 32) return false;
  // few examples: a workgroup still stages the whole filter, the patch-cotangent product wins
  // (B = 16 at 14 x 14: 25 against 23 us; from B = 32 on 26 against 27 and better)
  if (B * (ci / 32) * (((int64_t)h * w + 31) / 32) < 200) return false;
  return direct_shape(B, h, w, k, co, ci, true).ok;
}

hipError_t launch_conv_direct_reverse(const float *dz, const float *Wc, int64_t B, int32_t h, int32_t w,
                                      int32_t ci, int32_t k, int32_t co, float *din, hipStream_t stream) {
  if (!conv_direct_reverse_applies(dz, Wc, B, h, w, ci, k, co, din)) return hipErrorInvalidValue;
  const DirectShape s = direct_shape(B, h, w, k, co, ci, true);
  ConvDirectArgs a{};
  a.in = dz; a.Wc = Wc; a.out = din;
  a.h = h; a.w = w; a.k = k; a.ci = ci; a.co = co; a.q = co; a.o_total = ci;
  a.tiles = (h * w + 31) / 32; a.splits = s.splits; a.tc = s.tc; a.rows_max = s.rows_max;
  return launch_direct_nt<true>(a, s.nt, B * (ci / 32) * s.splits, s.smem, stream);
}

namespace {

size_t filter_smem(int h, int w, int k) {
  const size_t stage = ((size_t)(h + k - 1) * (w + k - 1) * 32 + (size_t)h * w * 32) * 4;
  return std::max(stage, (size_t)4 * 32 * 36 * 4);
}

template <int TT>
hipError_t launch_filter(const ConvFilterArgs &a, int64_t wgs, size_t smem, hipStream_t stream) {
  auto kern = conv_filter_direct_kernel<TT>;
  static bool attr_set = false;   // benign race: the attribute is idempotent
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds_limit());
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  PFG_KERNEL(kern, dim3((unsigned)wgs), dim3(kThreads), smem, stream, a);
  return hipGetLastError();
}

}  // namespace

bool conv_filter_direct_applies(const float *in, const float *dz, int64_t B, int32_t h, int32_t w, int32_t ci,
                                int32_t k, int32_t co, const float *dWc) {
  if (!in || !dz || !dWc || B < 1 || h < 2 || w < 2 || h % 2 || w % 2) return false;
  if (!aligned16(in) || !aligned16(dz) || !aligned16(dWc)) return false;
  if (ci < 32 || ci % 32 || co < 32 || co % 32 || (k != 3 && k != 5)) return false;
  if (B * (ci / 32) * (co / 32) > 0x7fffffffLL) return false;
  // a workgroup's time does not shrink with the batch (34 us at 14 x 14, 5 x 5): the batched product over
  // gathered patches is faster until the workgroups nearly fill the chip (B = 64: 38 against 45 us)
  if (B * (ci / 32) * (co / 32) < 224) return false;
  return filter_smem(h, w, k) <= (size_t)lds_limit();
}

int conv_filter_direct_parts(int32_t ci, int32_t co) { return (ci / 32) * (co / 32); }
int conv_filter_rows_parts(int32_t co) { return co / 32; }

hipError_t launch_conv_filter_direct(const float *in, const float *dz, int64_t B, int32_t h, int32_t w,
                                     int32_t ci, int32_t k, int32_t co, float *dWc, int streaming,
                                     float *sq_part, hipStream_t stream) {
  if (!conv_filter_direct_applies(in, dz, B, h, w, ci, k, co, dWc)) return hipErrorInvalidValue;
  ConvFilterArgs a{};
  a.in = in; a.dz = dz; a.dWc = dWc; a.h = h; a.w = w; a.k = k; a.ci = ci; a.co = co; a.streaming = streaming;
  a.sq_part = sq_part;
  const int64_t wgs = B * (ci / 32) * (co / 32);
  const size_t smem = filter_smem(h, w, k);
  return k == 3 ? launch_filter<3>(a, wgs, smem, stream) : launch_filter<7>(a, wgs, smem, stream);
}

namespace {

size_t filter_rows_smem(int h, int w, int k, int ci) {
  const int RS = ((w + k - 1) * ci) | 1;
  const size_t img = ((size_t)(h + k - 1) * RS + 3) & ~(size_t)3;
  const int mt = (k * k * ci + 31) / 32;
  return std::max((img + (size_t)h * w * 32) * 4, (size_t)4 * mt * 32 * 36 * 4);
}

template <int MT>
hipError_t launch_filter_rows(const ConvFilterArgs &a, int64_t wgs, size_t smem, hipStream_t stream) {
  auto kern = conv_filter_rows_kernel<MT>;
  static bool attr_set = false;   // benign race: the attribute is idempotent
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds_limit());
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  PFG_KERNEL(kern, dim3((unsigned)wgs), dim3(kThreads), smem, stream, a);
  return hipGetLastError();
}

}  // namespace

bool conv_filter_rows_applies(const float *in, const float *dz, int64_t B, int32_t h, int32_t w, int32_t ci,
                              int32_t k, int32_t co, const float *dWc) {
  if (!in || !dz || !dWc || B < 1 || h < 2 || w < 2 || h % 2 || w % 2 || k < 1 || k % 2 == 0 || ci < 1) return false;
  if (!aligned16(dz) || !aligned16(dWc)) return false;
  if ((int64_t)k * k * ci > 64 || co < 32 || co % 32) return false;
  if ((int64_t)h * w * 8 >= (1 << 24) || B * (co / 32) > 0x7fffffffLL) return false;
  // 12 us whatever the batch (28 x 28, 5 x 5): from 64 workgroups on it beats patch copy + small product
  if (B * (co / 32) < 64) return false;
  return filter_rows_smem(h, w, k, ci) <= (size_t)lds_limit();
}

hipError_t launch_conv_filter_rows(const float *in, const float *dz, int64_t B, int32_t h, int32_t w, int32_t ci,
                                   int32_t k, int32_t co, float *dWc, int streaming, float *sq_part,
                                   hipStream_t stream) {
  if (!conv_filter_rows_applies(in, dz, B, h, w, ci, k, co, dWc)) return hipErrorInvalidValue;
  ConvFilterArgs a{};
  a.in = in; a.dz = dz; a.dWc = dWc; a.h = h; a.w = w; a.k = k; a.ci = ci; a.co = co; a.streaming = streaming;
  a.sq_part = sq_part;
  const int64_t wgs = B * (co / 32);
  const size_t smem = filter_rows_smem(h, w, k, ci);
  return k * k * ci <= 32 ? launch_filter_rows<1>(a, wgs, smem, stream) : launch_filter_rows<2>(a, wgs, smem, stream);
}

}  // namespace pfg
