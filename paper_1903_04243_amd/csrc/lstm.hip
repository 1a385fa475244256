// Kernels of the unrolled LSTM that are not matrix products: the cell update, its reverse step on
// stacked cotangent rows, and the per-example weight gradient, which sums one outer product per
// time step because the same weights are used at every step.
//
// Cell (column blocks i, g, f, o of the [dx + H, 4H] weight matrix):
//   i = sigmoid(z_i), g = tanh(z_g), f = sigmoid(z_f), o = sigmoid(z_o)
//   c_t = f c_{t-1} + i g,   h_t = o tanh(c_t)
#include "common.h"

namespace pfg {

namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ float sigmoidf_(float v) { return 1.f / (1.f + __expf(-v)); }

// One thread per (b, k).  zx already holds x_t W_x + b; zh = h_{t-1} W_h (null at the first step,
// where the state is zero).  gates, cs and hs are [B, T, .] and receive step t.
__global__ __launch_bounds__(kThreads) void lstm_cell_forward_kernel(
    const float *zx, const float *zh, float *gates, float *cs, float *hs, int64_t B, int H, int T,
    int t) {
  const int64_t id = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (id >= B * H) return;
  const int64_t b = id / H;
  const int k = (int)(id - b * H);
  const float *zrow = zx + (b * T + t) * 4 * (int64_t)H;
  float zi = zrow[k], zg = zrow[H + k], zf = zrow[2 * H + k], zo = zrow[3 * H + k];
  if (zh) {
    const float *hrow = zh + b * 4 * (int64_t)H;
    zi += hrow[k]; zg += hrow[H + k]; zf += hrow[2 * H + k]; zo += hrow[3 * H + k];
  }
  const float i = sigmoidf_(zi), g = tanhf(zg), f = sigmoidf_(zf), o = sigmoidf_(zo);
  const float cprev = t > 0 ? cs[(b * T + t - 1) * (int64_t)H + k] : 0.f;
  const float c = f * cprev + i * g;
  float *grow = gates + (b * T + t) * 4 * (int64_t)H;
  grow[k] = i; grow[H + k] = g; grow[2 * H + k] = f; grow[3 * H + k] = o;
  cs[(b * T + t) * (int64_t)H + k] = c;
  hs[(b * T + t) * (int64_t)H + k] = o * tanhf(c);
}

// Reverse step t on stacked cotangent rows m = b * S + s.  The gate values and cell states belong
// to example b and are shared by its S rows (loop-invariant over s: not stacked, Section 3.4).
//   dc   += dh * o * (1 - tanh(c_t)^2)
//   dz_o  = dh * tanh(c_t) * o (1 - o)
//   dz_i  = dc * g * i (1 - i),  dz_g = dc * i * (1 - g^2),  dz_f = dc * c_{t-1} * f (1 - f)
//   dc_{t-1} = dc * f
// dh row m starts at dh + (m / S) * dh_batch_stride + (m % S) * H (batch stride 0: one block shared
// by all b).  dc is [rows, H], read unless first, and overwritten with dc_{t-1}.  dz row m starts
// at dz + m * dz_row_stride.
__global__ __launch_bounds__(kThreads) void lstm_cell_backward_kernel(
    const float *dh, int64_t dh_batch_stride, float *dc, int first, const float *gates,
    const float *cs, int64_t rows, int S, int H, int T, int t, float *dz, int64_t dz_row_stride) {
  const int64_t id = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (id >= rows * H) return;
  const int64_t m = id / H;
  const int k = (int)(id - m * H);
  const int64_t b = m / S, s = m - b * S;
  const float *grow = gates + (b * T + t) * 4 * (int64_t)H;
  const float i = grow[k], g = grow[H + k], f = grow[2 * H + k], o = grow[3 * H + k];
  const float tc = tanhf(cs[(b * T + t) * (int64_t)H + k]);
  const float cprev = t > 0 ? cs[(b * T + t - 1) * (int64_t)H + k] : 0.f;
  const float dhv = dh[b * dh_batch_stride + s * H + k];
  const float dct = (first ? 0.f : dc[m * H + k]) + dhv * o * (1.f - tc * tc);
  float *out = dz + m * dz_row_stride;
  out[k] = dct * g * i * (1.f - i);
  out[H + k] = dct * i * (1.f - g * g);
  out[2 * H + k] = dct * cprev * f * (1.f - f);
  out[3 * H + k] = dhv * tc * o * (1.f - o);
  dc[m * H + k] = dct * f;
}

// out[b, i, j] = sum_{t < nt} a[b * a_bs + t * a_ts + i] * g[b * g_bs + t * g_ts + j]
// (Section 3.4's both-operands-stacked matmul with a contraction over the time steps).  A lane keeps
// its four columns of all nt cotangent rows in registers and walks the rows i of its chunk; the a
// values of the chunk (uniform over the workgroup) are fetched once into LDS.  At most kPassSteps
// steps per launch; later launches add to the result.  One launch covers up to two row blocks of the same
// per-example matrix (here: the input rows and the recurrent rows of the LSTM weight gradient).
constexpr int kMaxSteps = 16;      // steps whose cotangent values a lane holds at a time
constexpr int kPassSteps = 64;     // steps of one launch (runs of kMaxSteps); more take further launches
constexpr int kRowsPerBlock = 4;     // measured best of 2 / 4 / 8 / 16 on the 384 x 1024 gradient

struct OuterSumPart {
  const float *a; int64_t a_bs, a_ts;
  const float *g; int64_t g_bs, g_ts;
  float *out;            // example b at out + b * out_bs, [d_in, d_out]
  int d_in, nt;
  int row_chunks;        // ceil(d_in / kRowsPerBlock)
};

struct OuterSumArgs {
  OuterSumPart part[2];
  int nparts;
  int64_t out_bs;
  int d_out;
  int accumulate;        // add to out instead of overwriting it
  int vec;               // d_out % 4 == 0 and g, out 16-byte aligned with aligned strides
};

// NT: the steps of a pass rounded up to a multiple of 4 (a step past nt holds zeros), so that short
// loops over the steps pay for the steps they have.
template <int NT>
__global__ __launch_bounds__(kThreads) void outer_sum_kernel(const OuterSumArgs p) {
  __shared__ __align__(16) float a_s[kRowsPerBlock][NT];
  const int64_t b = blockIdx.y;
  const int col_chunks = (p.d_out + 4 * kThreads - 1) / (4 * kThreads);
  const int cchunk = blockIdx.x % col_chunks;
  int rchunk = blockIdx.x / col_chunks;
  const bool second = (p.nparts > 1) && (rchunk >= p.part[0].row_chunks);
  const OuterSumPart &q = p.part[second ? 1 : 0];
  if (second) rchunk -= p.part[0].row_chunks;
  const int i0 = rchunk * kRowsPerBlock;
  const int nrows = min(q.d_in - i0, kRowsPerBlock);
  const float *a = q.a + b * q.a_bs;
  const float *g = q.g + b * q.g_bs;
  float *out = q.out + b * p.out_bs;
  // the chunk's a values: adjacent lanes fetch adjacent rows of one step; kept step-fastest
  for (int e = threadIdx.x; e < NT * kRowsPerBlock; e += kThreads) {
    const int t = e / kRowsPerBlock, r = e % kRowsPerBlock;
    a_s[r][t] = (t < q.nt && r < nrows) ? a[t * q.a_ts + i0 + r] : 0.f;
  }
  __syncthreads();
  const int j = (cchunk * kThreads + threadIdx.x) * 4;
  if (j >= p.d_out) return;
  f32x4 gv[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    gv[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (t < q.nt) {
      if (p.vec) {
        gv[t] = *reinterpret_cast<const f32x4 *>(g + t * q.g_ts + j);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (j + e < p.d_out) gv[t][e] = g[t * q.g_ts + j + e];
      }
    }
  }
  for (int r = 0; r < nrows; ++r) {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t4 = 0; t4 < NT; t4 += 4) {
      const f32x4 av = *reinterpret_cast<const f32x4 *>(&a_s[r][t4]);
#pragma unroll
      for (int e = 0; e < 4; ++e) acc += av[e] * gv[t4 + e];           // steps past nt hold zeros
    }
    float *o = out + (int64_t)(i0 + r) * p.d_out + j;
    if (p.vec) {
      if (p.accumulate)
        *reinterpret_cast<f32x4 *>(o) = *reinterpret_cast<const f32x4 *>(o) + acc;
      else
        __builtin_nontemporal_store(acc, reinterpret_cast<f32x4 *>(o));
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (j + e < p.d_out) o[e] = p.accumulate ? o[e] + acc[e] : acc[e];
    }
  }
}

// More than kMaxSteps steps in one launch: walked in runs of kMaxSteps steps with the sums of the
// workgroup's rows kept in registers, so that the result is still written once.  (Kept apart from
// the kernel above, which is 3 % faster on a single run.)
__global__ __launch_bounds__(kThreads) void outer_sum_runs_kernel(const OuterSumArgs p) {
  constexpr int NT = kMaxSteps, NTL = kPassSteps;
  __shared__ __align__(16) float a_s[kRowsPerBlock][NTL];
  const int64_t b = blockIdx.y;
  const int col_chunks = (p.d_out + 4 * kThreads - 1) / (4 * kThreads);
  const int cchunk = blockIdx.x % col_chunks;
  int rchunk = blockIdx.x / col_chunks;
  const bool second = (p.nparts > 1) && (rchunk >= p.part[0].row_chunks);
  const OuterSumPart &q = p.part[second ? 1 : 0];
  if (second) rchunk -= p.part[0].row_chunks;
  const int i0 = rchunk * kRowsPerBlock;
  const int nrows = min(q.d_in - i0, kRowsPerBlock);
  const float *a = q.a + b * q.a_bs;
  const float *g = q.g + b * q.g_bs;
  float *out = q.out + b * p.out_bs;
  // the chunk's a values: adjacent lanes fetch adjacent rows of one step; kept step-fastest
  for (int e = threadIdx.x; e < NTL * kRowsPerBlock; e += kThreads) {
    const int t = e / kRowsPerBlock, r = e % kRowsPerBlock;
    a_s[r][t] = (t < q.nt && r < nrows) ? a[t * q.a_ts + i0 + r] : 0.f;
  }
  __syncthreads();
  const int j = (cchunk * kThreads + threadIdx.x) * 4;
  if (j >= p.d_out) return;
  f32x4 acc[kRowsPerBlock];
#pragma unroll
  for (int r = 0; r < kRowsPerBlock; ++r) acc[r] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int t0 = 0; t0 < NTL && t0 < q.nt; t0 += NT) {
    f32x4 gv[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      gv[t] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (t0 + t < q.nt) {
        if (p.vec) {
          gv[t] = *reinterpret_cast<const f32x4 *>(g + (t0 + t) * q.g_ts + j);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (j + e < p.d_out) gv[t][e] = g[(t0 + t) * q.g_ts + j + e];
        }
      }
    }
#pragma unroll
    for (int r = 0; r < kRowsPerBlock; ++r) {
#pragma unroll
      for (int t4 = 0; t4 < NT; t4 += 4) {
        const f32x4 av = *reinterpret_cast<const f32x4 *>(&a_s[r][t0 + t4]);
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[r] += av[e] * gv[t4 + e];      // steps past nt hold zeros
      }
    }
  }
#pragma unroll
  for (int r = 0; r < kRowsPerBlock; ++r) {
    if (r >= nrows) break;
    float *o = out + (int64_t)(i0 + r) * p.d_out + j;
    if (p.vec) {
      if (p.accumulate)
        *reinterpret_cast<f32x4 *>(o) = *reinterpret_cast<const f32x4 *>(o) + acc[r];
      else
        __builtin_nontemporal_store(acc[r], reinterpret_cast<f32x4 *>(o));
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (j + e < p.d_out) o[e] = p.accumulate ? o[e] + acc[r][e] : acc[r][e];
    }
  }
}

// out[b, j] = sum_t g[b, t, j].  One workgroup per (b, group of up to 64 columns); its threads form
// 256 / columns row slots that each add every (256 / columns)-th row, then the slots are added in a
// fixed order.  Rows are read 128 or 256 bytes at a time by adjacent lanes.
// With pieces > 1 the third grid index selects a piece of the T rows and the result is a partial
// sum, written as row (b, piece) of out [B, pieces, d] (a second pass of the same kernel adds them).
__global__ __launch_bounds__(kThreads) void sum_steps_kernel(const float *g, int T, int d, int cols,
                                                             int pieces, float *out) {
  __shared__ float part[kThreads];
  const int64_t b = blockIdx.y;
  const int piece = blockIdx.z;
  const int per = (T + pieces - 1) / pieces;
  const int t0 = piece * per, t1 = min(T, t0 + per);
  const int j0 = blockIdx.x * cols;
  const int slots = kThreads / cols;
  const int slot = threadIdx.x / cols, j = j0 + threadIdx.x % cols;
  float s = 0.f;
  if (j < d)
    for (int t = t0 + slot; t < t1; t += slots) s += g[(b * T + t) * (int64_t)d + j];
  part[threadIdx.x] = s;
  __syncthreads();
  if (threadIdx.x < cols && j < d) {
    float total = 0.f;
    for (int r = 0; r < slots; ++r) total += part[r * cols + threadIdx.x];
    out[(b * pieces + piece) * (int64_t)d + j] = total;
  }
}

// One wave's share of sum_k a[k] * b[k]: lanes stride over the n values (16 bytes at a time when both
// rows allow it); the caller adds the lanes up.
__device__ __forceinline__ float lane_dot(const float *a, const float *b, int n, int lane) {
  float s = 0.f;
  if (n % 4 == 0 && ((reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b)) & 15) == 0) {
    for (int k = 4 * lane; k < n; k += 256) {
      const f32x4 x = *reinterpret_cast<const f32x4 *>(a + k), y = *reinterpret_cast<const f32x4 *>(b + k);
      s += x[0] * y[0] + x[1] * y[1] + x[2] * y[2] + x[3] * y[3];
    }
  } else {
    for (int k = lane; k < n; k += 64) s += a[k] * b[k];
  }
  return s;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// Squared norms of one example's LSTM gradient without the gradient.  The same W acts at every step,
// dW[b] = sum_t u_t^T dz_t with u_t = [x_t, h_{t-1}], so
//     |dW[b]|^2 = sum_{t, t'} (u_t . u_t') (dz_t . dz_t')      and      |db[b]|^2 = sum_{t, t'} dz_t . dz_t':
// two T x T Gram matrices per example instead of a [dx + H, 4H] matrix.  The readout gradient is an
// outer product: |dWout[b]|^2 = |h_T|^2 |dy|^2, |dbout[b]|^2 = |dy|^2.  One workgroup per example; a
// wave takes every sixteenth pair (t <= t'), everything is added in a fixed order.
constexpr int kMaxNormSteps = 64;

constexpr int kNormThreads = 1024;     // 16 waves: the pairs are many short, latency-bound dot products

__global__ __launch_bounds__(kNormThreads) void lstm_grad_sqnorms_kernel(const float *X, const float *hs,
                                                                         const float *dz, const float *gy,
                                                                         int T, int dx, int H, int dy,
                                                                         float *sq, float *norm) {
  __shared__ float pw[kMaxNormSteps * (kMaxNormSteps + 1) / 2], pb[kMaxNormSteps * (kMaxNormSteps + 1) / 2];
  __shared__ float tail[2];
  const int64_t b = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float *xb = X + b * T * (int64_t)dx, *hb = hs + b * T * (int64_t)H, *zb = dz + b * T * (int64_t)(4 * H);
  const int pairs = T * (T + 1) / 2;
  for (int p = wave; p < pairs; p += kNormThreads / 64) {
    int t = 0, r = p;
    while (r >= T - t) { r -= T - t; ++t; }
    const int u = t + r;                                   // the pair (t, u), t <= u
    float gz = lane_dot(zb + (int64_t)t * 4 * H, zb + (int64_t)u * 4 * H, 4 * H, lane);
    float gu = lane_dot(xb + (int64_t)t * dx, xb + (int64_t)u * dx, dx, lane);
    if (t >= 1) gu += lane_dot(hb + (int64_t)(t - 1) * H, hb + (int64_t)(u - 1) * H, H, lane);   // h_0 = 0
    gz = wave_sum(gz);
    gu = wave_sum(gu);
    if (lane == 0) {
      const float twice = (t == u) ? 1.f : 2.f;           // the pair (u, t) contributes the same
      pw[p] = twice * gu * gz;
      pb[p] = twice * gz;
    }
  }
  if (wave == 0) {
    const float *hT = hb + (int64_t)(T - 1) * H;
    const float v = wave_sum(lane_dot(hT, hT, H, lane));
    if (lane == 0) tail[0] = v;
  } else if (wave == 1) {
    const float *g = gy + b * dy;
    const float v = wave_sum(lane_dot(g, g, dy, lane));
    if (lane == 0) tail[1] = v;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float sw = 0.f, sb = 0.f;
    for (int p = 0; p < pairs; ++p) {
      sw += pw[p];
      sb += pb[p];
    }
    const float so = tail[0] * tail[1], sbo = tail[1];
    if (sq) {
      sq[4 * b] = sw; sq[4 * b + 1] = sb; sq[4 * b + 2] = so; sq[4 * b + 3] = sbo;
    }
    if (norm) norm[b] = sqrtf(sw + sb + so + sbo);
  }
}

inline unsigned blocks_for(int64_t n) { return (unsigned)((n + kThreads - 1) / kThreads); }

}  // namespace

hipError_t launch_lstm_cell_forward(const float *zx, const float *zh, float *gates, float *cs,
                                    float *hs, int64_t B, int32_t H, int32_t T, int32_t t,
                                    hipStream_t stream) {
  if (B <= 0) return hipSuccess;
  PFG_KERNEL(lstm_cell_forward_kernel, dim3(blocks_for(B * H)), dim3(kThreads), 0, stream, zx, zh,
             gates, cs, hs, B, H, T, t);
  return hipGetLastError();
}

hipError_t launch_lstm_cell_backward(const float *dh, int64_t dh_batch_stride, float *dc, int32_t first,
                                     const float *gates, const float *cs, int64_t rows, int32_t S,
                                     int32_t H, int32_t T, int32_t t, float *dz, int64_t dz_row_stride,
                                     hipStream_t stream) {
  if (rows <= 0) return hipSuccess;
  PFG_KERNEL(lstm_cell_backward_kernel, dim3(blocks_for(rows * H)), dim3(kThreads), 0, stream, dh,
             dh_batch_stride, dc, first, gates, cs, rows, S, H, T, t, dz, dz_row_stride);
  return hipGetLastError();
}

hipError_t launch_outer_sum(const OuterSumJob *jobs, int njobs, int64_t B, int32_t d_out,
                            int64_t out_bs, hipStream_t stream) {
  if (B <= 0 || d_out <= 0 || njobs <= 0) return hipSuccess;
  if (njobs > 2) return hipErrorInvalidValue;
  auto aligned = [](const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
  int vec = d_out % 4 == 0 && out_bs % 4 == 0;
  int max_nt = 0;
  for (int k = 0; k < njobs; ++k) {
    vec = vec && aligned(jobs[k].g) && aligned(jobs[k].out) && jobs[k].g_bs % 4 == 0 &&
          jobs[k].g_ts % 4 == 0;
    max_nt = jobs[k].nt > max_nt ? jobs[k].nt : max_nt;
  }
  const int col_chunks = (d_out + 4 * kThreads - 1) / (4 * kThreads);
  for (int64_t b0 = 0; b0 < B; b0 += 32768) {          // the second grid index holds 65535 at most
    const int64_t nb = B - b0 < 32768 ? B - b0 : 32768;
    int t0 = 0;
    do {
      OuterSumArgs p{};
      int row_chunks = 0;
      for (int k = 0; k < njobs; ++k) {
        const OuterSumJob &jb = jobs[k];
        int nt = jb.nt - t0;                           // a job with no step left contributes zeros
        nt = nt < 0 ? 0 : (nt > kPassSteps ? kPassSteps : nt);
        OuterSumPart &q = p.part[k];
        q.a = jb.a + b0 * jb.a_bs + (int64_t)t0 * jb.a_ts; q.a_bs = jb.a_bs; q.a_ts = jb.a_ts;
        q.g = jb.g + b0 * jb.g_bs + (int64_t)t0 * jb.g_ts; q.g_bs = jb.g_bs; q.g_ts = jb.g_ts;
        q.out = jb.out + b0 * out_bs;
        q.d_in = jb.d_in; q.nt = nt;
        q.row_chunks = (jb.d_in + kRowsPerBlock - 1) / kRowsPerBlock;
        row_chunks += q.row_chunks;
      }
      p.nparts = njobs; p.out_bs = out_bs; p.d_out = d_out; p.accumulate = t0 > 0; p.vec = vec;
      const dim3 grid((unsigned)(col_chunks * row_chunks), (unsigned)nb);
      const int pass_nt = max_nt - t0;
      if (pass_nt <= 4)       PFG_KERNEL(outer_sum_kernel<4>, grid, dim3(kThreads), 0, stream, p);
      else if (pass_nt <= 8)  PFG_KERNEL(outer_sum_kernel<8>, grid, dim3(kThreads), 0, stream, p);
      else if (pass_nt <= 12) PFG_KERNEL(outer_sum_kernel<12>, grid, dim3(kThreads), 0, stream, p);
      else if (pass_nt <= kMaxSteps) PFG_KERNEL(outer_sum_kernel<kMaxSteps>, grid, dim3(kThreads), 0, stream, p);
      else                    PFG_KERNEL(outer_sum_runs_kernel, grid, dim3(kThreads), 0, stream, p);
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
      t0 += kPassSteps;
    } while (t0 < max_nt);
  }
  return hipSuccess;
}

hipError_t launch_lstm_grad_sqnorms(const float *X, const float *hs, const float *dz, const float *gy,
                                    int64_t B, int32_t T, int32_t dx, int32_t H, int32_t dy, float *sq,
                                    float *norm, hipStream_t stream) {
  if (B <= 0) return hipSuccess;
  if (T > kMaxNormSteps || B > 0x7fffffffLL) return hipErrorInvalidValue;
  PFG_KERNEL(lstm_grad_sqnorms_kernel, dim3((unsigned)B), dim3(kNormThreads), 0, stream, X, hs, dz, gy, T, dx, H,
             dy, sq, norm);
  return hipGetLastError();
}

hipError_t launch_sum_steps(const float *g, int64_t B, int32_t T, int32_t d, float *out,
                            float *scratch, hipStream_t stream) {
  if (B <= 0 || d <= 0) return hipSuccess;
  int cols = 64;                       // 64, 32 or 16 columns per workgroup, not more than needed
  while (cols > 16 && cols / 2 >= d) cols /= 2;
  const unsigned groups = (unsigned)((d + cols - 1) / cols);
  // many rows and few workgroups: sum kSumPieces pieces of the rows separately first
  const int pieces = (scratch && T >= 128 && B * groups < 2048) ? kSumPieces : 1;
  for (int64_t b0 = 0; b0 < B; b0 += 32768) {
    const int64_t nb = B - b0 < 32768 ? B - b0 : 32768;
    float *first_out = pieces > 1 ? scratch : out + b0 * d;
    PFG_KERNEL(sum_steps_kernel, dim3(groups, (unsigned)nb, (unsigned)pieces), dim3(kThreads), 0, stream,
               g + b0 * T * (int64_t)d, T, d, cols, pieces, first_out);
    if (pieces > 1)
      PFG_KERNEL(sum_steps_kernel, dim3(groups, (unsigned)nb, 1u), dim3(kThreads), 0, stream, scratch,
                 pieces, d, cols, 1, out + b0 * d);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace pfg
