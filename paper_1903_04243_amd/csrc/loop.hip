// Kernels of the sequential while loop inside a parallel-for (Section 3.7).  The converted loop
// keeps the list I of the iterations that are still active; every trip evaluates the condition on
// the rows of I only, keeps the rows for which it holds (in increasing order of the iteration
// index), and runs the body on those.  Here the list, its length and the per-iteration trip
// counts stay in device memory: the host enqueues a fixed number of trips, each kernel reads the
// live length itself and has nothing to do once the list is empty, so the loop neither
// synchronises with the host nor depends on the data in its launch sequence.
//
// The loop of this library's LSTM: iteration i runs while  t < len_i  and
// halt_c + <h_i, halt_w> <= 0  (the cap on the number of trips is the number of trips enqueued).
#include "common.h"

namespace pfg {

namespace {

constexpr int kGroup = 32;       // rows whose kept flags are counted together
constexpr int kPlace = 1024;     // rows per workgroup of the placing kernel (a multiple of kGroup)

// I[m] = m, meta = {B, 0}, steps[i] = max_steps (a row that is never dropped ran to the cap), trips = 0
__global__ __launch_bounds__(256) void while_init_kernel(int32_t *I, int32_t *meta, int32_t *steps, int32_t *trips,
                                                         int B, int max_steps) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < B) {
    I[i] = i;
    steps[i] = max_steps;
  }
  if (i == 0) {
    meta[0] = B;
    meta[1] = 0;
    if (trips) *trips = 0;
  }
}

// The condition of trip t on the rows of the active list: flags[m] = 1 if iteration I[m] goes on.
// An iteration that stops here has made t trips: steps[I[m]] = t.  cnt[m / kGroup] = kept rows of the
// group.  16 lanes share a row of h (fixed summation order); a workgroup takes 32 rows in two passes.
// Token ranges come from seq_offsets [B + 1]; a range that does not lie inside [0, total_tokens] is
// cut to it, so that whatever the array holds no token row outside X is ever used.
__global__ __launch_bounds__(256) void while_flags_kernel(const int32_t *I, const int32_t *meta, int t,
                                                          const int32_t *seq_offsets, int total_tokens,
                                                          const float *h, int H, const float *w, float c0,
                                                          int32_t *flags, int32_t *cnt, int32_t *steps) {
  const int l = meta[0];
  if (blockIdx.x * kGroup >= l) return;
  __shared__ int s_cnt;
  if (threadIdx.x == 0) s_cnt = 0;
  __syncthreads();
  const int slot = threadIdx.x >> 4, l16 = threadIdx.x & 15;
  const bool vec = w && ((reinterpret_cast<uintptr_t>(h) | reinterpret_cast<uintptr_t>(w)) & 15) == 0 && H % 4 == 0;
  int mine = 0;
  for (int pass = 0; pass < kGroup / 16; ++pass) {
    const int m = blockIdx.x * kGroup + pass * 16 + slot;
    const int i = (m < l) ? I[m] : 0;
    float s = 0.f;
    if (m < l && w) {
      const float *row = h + (int64_t)i * H;
      if (vec) {
        for (int k = 4 * l16; k < H; k += 64) {
          const f32x4 a = *reinterpret_cast<const f32x4 *>(row + k);
          const f32x4 b = *reinterpret_cast<const f32x4 *>(w + k);
          s += a[0] * b[0] + a[1] * b[1] + a[2] * b[2] + a[3] * b[3];
        }
      } else {
        for (int k = l16; k < H; k += 16) s += row[k] * w[k];
      }
    }
#pragma unroll
    for (int off = 8; off > 0; off >>= 1) s += __shfl_xor(s, off, 16);
    if (l16 == 0 && m < l) {
      const int lo = seq_offsets[i], hi = min(seq_offsets[i + 1], total_tokens);
      const int len = (lo >= 0 && hi > lo) ? hi - lo : 0;
      const int f = (t < len && s + c0 <= 0.f) ? 1 : 0;
      flags[m] = f;
      if (!f) steps[i] = t;
      mine += f;
    }
  }
  if (l16 == 0 && mine) atomicAdd(&s_cnt, mine);      // integers: the order does not matter
  __syncthreads();
  if (threadIdx.x == 0) cnt[blockIdx.x] = s_cnt;
}

// blk[b] = sum of the group counts of the kPlace rows one placing workgroup takes (many rows only)
__global__ __launch_bounds__(256) void while_block_counts_kernel(const int32_t *cnt, const int32_t *meta,
                                                                 int32_t *blk) {
  constexpr int kPer = kPlace / kGroup;
  const int l = meta[0];
  const int ngroups = (l + kGroup - 1) / kGroup, nblocks = (l + kPlace - 1) / kPlace;
  const int b = blockIdx.x * 256 + threadIdx.x;
  if (b >= nblocks) return;
  int s = 0;
  for (int g = b * kPer; g < min((b + 1) * kPer, ngroups); ++g) s += cnt[g];
  blk[b] = s;
}

// I_next = the kept rows of I, order preserved; meta_next = {their number, 0}.  A workgroup places
// kPlace consecutive rows of the list: it adds up the counts in front of them (group counts, or
// block counts when blk is given), ranks its own rows with a ballot per wave, and writes.
__global__ __launch_bounds__(kPlace) void while_place_kernel(const int32_t *flags, const int32_t *cnt,
                                                             const int32_t *blk, const int32_t *I,
                                                             const int32_t *meta, int32_t *I_next,
                                                             int32_t *meta_next, int32_t *trips, int t) {
  constexpr int kWaves = kPlace / 64;
  __shared__ int s_before[kWaves], s_total[kWaves], s_wave[kWaves];
  const int l = meta[0];
  if (blockIdx.x * kPlace >= l && blockIdx.x != 0) return;       // workgroup 0 always writes meta_next
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int32_t *c = blk ? blk : cnt;
  const int per = blk ? kPlace : kGroup;
  const int ncounts = (l + per - 1) / per;
  const int first = blockIdx.x * (kPlace / per);
  int before = 0, total = 0;
  for (int g = tid; g < ncounts; g += kPlace) {
    const int v = c[g];
    total += v;
    if (g < first) before += v;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    before += __shfl_xor(before, off, 64);
    total += __shfl_xor(total, off, 64);
  }
  const int m = blockIdx.x * kPlace + tid;
  const int f = (m < l) ? flags[m] : 0;
  const unsigned long long set = __ballot(f != 0);
  const int rank_in_wave = __popcll(set & ((1ull << lane) - 1ull));
  if (lane == 0) {
    s_before[wave] = before;
    s_total[wave] = total;
    s_wave[wave] = __popcll(set);
  }
  __syncthreads();
  int kept_before = 0, kept = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    kept_before += s_before[w];
    kept += s_total[w];
    if (w < wave) kept_before += s_wave[w];
  }
  if (f) I_next[kept_before + rank_in_wave] = I[m];
  if (blockIdx.x == 0 && tid == 0) {
    meta_next[0] = kept;
    meta_next[1] = 0;
    if (trips && kept > 0) *trips = t + 1;
  }
}

// h_out[i, :] = the state iteration i left the loop with: zero after no trip, else the buffer its
// last trip wrote (trip t writes buffer t % 2).
__global__ __launch_bounds__(256) void while_state_kernel(const int32_t *steps, const float *h_even,
                                                          const float *h_odd, int64_t B, int H, float *h_out) {
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= B * H) return;
  const int s = steps[e / H];
  h_out[e] = s <= 0 ? 0.f : (((s - 1) & 1) ? h_odd[e] : h_even[e]);
}


// Reverse trip t of the loop on the rows that made trip t (the list the forward pass kept for it).
// Row m of the list is iteration i = I[m]; its token row of trip t is r = first token of i + t.
//   dc    = dc[i] + dh[i] * o * (1 - tanh(c_t)^2)
//   dz_o  = dh[i] * tanh(c_t) * o (1 - o)
//   dz_i  = dc * g * i (1 - i),  dz_g = dc * i * (1 - g^2),  dz_f = dc * c_{t-1} * f (1 - f)
//   dc[i] = dc * f
// dz goes to token row r of dz_tok (for the sums over an iteration's trips) and to row m of dz_packed
// (the operand of the product that carries dh to trip t - 1).  An iteration that has not started its
// reverse sweep yet is in no list: its dh keeps the seed and its dc the zero it was given.
__global__ __launch_bounds__(256) void while_cell_backward_kernel(const int32_t *I, const int32_t *meta, int t,
                                                                  const int32_t *seq_offsets, int total_tokens,
                                                                  const float *gates_tok, const float *c_tok,
                                                                  const float *dh, float *dc, float *dz_tok,
                                                                  float *dz_packed, int H) {
  const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t m = id / H;
  if (m >= meta[0]) return;
  const int k = (int)(id - m * H);
  const int64_t i = I[m];
  const int64_t r = (int64_t)seq_offsets[i] + t;
  if (seq_offsets[i] < 0 || r >= total_tokens) return;      // cannot happen for a list the forward pass built
  const float *grow = gates_tok + r * 4 * H;
  const float gi = grow[k], gg = grow[H + k], gf = grow[2 * H + k], go = grow[3 * H + k];
  const float tc = tanhf(c_tok[r * H + k]);
  const float cprev = t > 0 ? c_tok[(r - 1) * H + k] : 0.f;
  const float dhv = dh[i * H + k];
  const float dct = dc[i * H + k] + dhv * go * (1.f - tc * tc);
  const float zi = dct * gg * gi * (1.f - gi), zg = dct * gi * (1.f - gg * gg);
  const float zf = dct * cprev * gf * (1.f - gf), zo = dhv * tc * go * (1.f - go);
  float *a = dz_tok + r * 4 * H, *b = dz_packed + m * 4 * H;
  a[k] = zi; a[H + k] = zg; a[2 * H + k] = zf; a[3 * H + k] = zo;
  b[k] = zi; b[H + k] = zg; b[2 * H + k] = zf; b[3 * H + k] = zo;
  dc[i * H + k] = dct * gf;
}

// Per-iteration sums over the trips an iteration made (the same W acts in every trip, so an
// iteration's gradient is the sum of its trips' outer products; different iterations stay apart):
//   dW[b, 0:dx, :]      = sum_{t < T_b} x[r_b + t, :]^T     dz[r_b + t, :]
//   dW[b, dx:dx+H, :]   = sum_{1 <= t < T_b} h[r_b + t - 1, :]^T dz[r_b + t, :]      (h before trip 0 is zero)
//   db[b, :]            = sum_{t < T_b} dz[r_b + t, :]
// with r_b the iteration's first token row and T_b = steps[b] its trip count (both from device
// memory, cut to the iteration's token range).  A workgroup takes kRaggedRows rows of one iteration's
// matrix and up to 1024 columns; a lane keeps its four columns of kRaggedRun cotangent rows in
// registers at a time and the a-values of the run go through LDS (uniform over the workgroup).  The
// result is written once, also when T_b = 0 (zeros).
constexpr int kRaggedRows = 8;
constexpr int kRaggedRun = 16;

struct RaggedSumArgs {
  const float *x; int dx;
  const float *h_tok; int H;
  const float *dz_tok;           // [tokens, d_out]
  const int32_t *seq_offsets;    // [B + 1]
  const int32_t *steps;          // [B]
  int total_tokens;
  float *dW;                     // [B, dx + H, d_out] or nullptr
  float *db;                     // [B, d_out] or nullptr
  int d_out;
  int vec;                       // 16-byte stores allowed (alignment of dW, db)
};

__global__ __launch_bounds__(256) void outer_sum_ragged_kernel(const RaggedSumArgs p) {
  __shared__ __align__(16) float a_s[kRaggedRows][kRaggedRun];
  const int64_t b = blockIdx.y;
  const int col_chunks = (p.d_out + 1023) / 1024;
  const int cchunk = blockIdx.x % col_chunks;
  int rchunk = blockIdx.x / col_chunks;
  const int chunks_x = (p.dx + kRaggedRows - 1) / kRaggedRows, chunks_h = (p.H + kRaggedRows - 1) / kRaggedRows;
  // part 0: input rows, 1: recurrent rows, 2: the bias row
  int part = 0;
  if (!p.dW) { part = 2; rchunk = 0; }
  else if (rchunk >= chunks_x + chunks_h) { part = 2; rchunk = 0; }
  else if (rchunk >= chunks_x) { part = 1; rchunk -= chunks_x; }
  const int d_in = part == 0 ? p.dx : part == 1 ? p.H : 1;
  const int i0 = rchunk * kRaggedRows;
  const int nrows = min(d_in - i0, kRaggedRows);
  const int lo = p.seq_offsets[b], hi = min(p.seq_offsets[b + 1], p.total_tokens);
  const int len = (lo >= 0 && hi > lo) ? hi - lo : 0;
  const int nt = max(0, min(p.steps[b], len));
  const int j = (cchunk * 256 + threadIdx.x) * 4;
  f32x4 acc[kRaggedRows];
#pragma unroll
  for (int r = 0; r < kRaggedRows; ++r) acc[r] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int t0 = 0; t0 < nt; t0 += kRaggedRun) {
    __syncthreads();                       // the previous run's values have been used
    if (threadIdx.x < kRaggedRows * kRaggedRun) {
      const int tt = threadIdx.x / kRaggedRows, r = threadIdx.x % kRaggedRows;
      const int t = t0 + tt;
      float v = 0.f;
      if (t < nt && r < nrows) {
        if (part == 0) v = p.x[(int64_t)(lo + t) * p.dx + i0 + r];
        else if (part == 1) v = t > 0 ? p.h_tok[(int64_t)(lo + t - 1) * p.H + i0 + r] : 0.f;
        else v = 1.f;
      }
      a_s[r][tt] = v;
    }
    __syncthreads();
    if (j < p.d_out) {
      f32x4 gv[kRaggedRun];
#pragma unroll
      for (int tt = 0; tt < kRaggedRun; ++tt) {
        gv[tt] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (t0 + tt < nt) {
          const float *g = p.dz_tok + (int64_t)(lo + t0 + tt) * p.d_out + j;
          if (j + 4 <= p.d_out && (p.d_out & 3) == 0) {
            gv[tt] = *reinterpret_cast<const f32x4 *>(g);
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (j + e < p.d_out) gv[tt][e] = g[e];
          }
        }
      }
#pragma unroll
      for (int r = 0; r < kRaggedRows; ++r) {
#pragma unroll
        for (int t4 = 0; t4 < kRaggedRun; t4 += 4) {
          const f32x4 av = *reinterpret_cast<const f32x4 *>(&a_s[r][t4]);
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[r] += av[e] * gv[t4 + e];
        }
      }
    }
  }
  if (j >= p.d_out) return;
  float *out = part == 2 ? p.db + b * (int64_t)p.d_out
                         : p.dW + (b * (int64_t)(p.dx + p.H) + (part == 1 ? p.dx : 0) + i0) * p.d_out;
#pragma unroll
  for (int r = 0; r < kRaggedRows; ++r) {
    if (r >= nrows) break;
    float *o = out + (int64_t)r * p.d_out + j;
    if (p.vec && j + 4 <= p.d_out) {
      __builtin_nontemporal_store(acc[r], reinterpret_cast<f32x4 *>(o));
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (j + e < p.d_out) o[e] = acc[r][e];
    }
  }
}

}  // namespace

int64_t while_count_entries(int64_t B) { return (B + kGroup - 1) / kGroup + (B + kPlace - 1) / kPlace; }

hipError_t launch_while_init(int32_t *I, int32_t *meta, int32_t *steps, int32_t *trips, int32_t B,
                             int32_t max_steps, hipStream_t stream) {
  PFG_KERNEL(while_init_kernel, dim3((unsigned)((B + 255) / 256)), dim3(256), 0, stream, I, meta, steps, trips, B,
             max_steps);
  return hipGetLastError();
}

hipError_t launch_while_select(const int32_t *I, const int32_t *meta, int32_t t, const int32_t *seq_offsets,
                               int32_t total_tokens, const float *h, int32_t H, const float *w, float c0,
                               int32_t B, int32_t *flags, int32_t *cnt, int32_t *I_next, int32_t *meta_next,
                               int32_t *steps, int32_t *trips, hipStream_t stream) {
  const int ngroups = (B + kGroup - 1) / kGroup, nblocks = (B + kPlace - 1) / kPlace;
  PFG_KERNEL(while_flags_kernel, dim3((unsigned)ngroups), dim3(256), 0, stream, I, meta, t, seq_offsets,
             total_tokens, h, H, w, c0, flags, cnt, steps);
  int32_t *blk = nullptr;
  if (B > (1 << 16)) {
    blk = cnt + ngroups;
    PFG_KERNEL(while_block_counts_kernel, dim3((unsigned)((nblocks + 255) / 256)), dim3(256), 0, stream, cnt, meta,
               blk);
  }
  PFG_KERNEL(while_place_kernel, dim3((unsigned)nblocks), dim3(kPlace), 0, stream, flags, cnt, blk, I, meta, I_next,
             meta_next, trips, t);
  return hipGetLastError();
}

hipError_t launch_while_state(const int32_t *steps, const float *h_even, const float *h_odd, int64_t B, int32_t H,
                              float *h_out, hipStream_t stream) {
  const int64_t n = B * H;
  PFG_KERNEL(while_state_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, steps, h_even, h_odd, B, H,
             h_out);
  return hipGetLastError();
}

hipError_t launch_while_cell_backward(const int32_t *I, const int32_t *meta, int32_t t, const int32_t *seq_offsets,
                                      int32_t total_tokens, const float *gates_tok, const float *c_tok,
                                      const float *dh, float *dc, float *dz_tok, float *dz_packed, int64_t B,
                                      int32_t H, hipStream_t stream) {
  const int64_t n = B * H;
  PFG_KERNEL(while_cell_backward_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, I, meta, t,
             seq_offsets, total_tokens, gates_tok, c_tok, dh, dc, dz_tok, dz_packed, H);
  return hipGetLastError();
}

hipError_t launch_outer_sum_ragged(const float *x, int32_t dx, const float *h_tok, int32_t H, const float *dz_tok,
                                   const int32_t *seq_offsets, const int32_t *steps, int32_t total_tokens, int64_t B,
                                   float *dW, float *db, hipStream_t stream) {
  if (!dW && !db) return hipSuccess;
  if (B > 65535) return hipErrorInvalidConfiguration;
  RaggedSumArgs p{};
  p.x = x; p.dx = dx; p.h_tok = h_tok; p.H = H; p.dz_tok = dz_tok;
  p.seq_offsets = seq_offsets; p.steps = steps; p.total_tokens = total_tokens;
  p.dW = dW; p.db = db; p.d_out = 4 * H;
  p.vec = (((reinterpret_cast<uintptr_t>(dW) | reinterpret_cast<uintptr_t>(db)) & 15) == 0) ? 1 : 0;
  const int col_chunks = (p.d_out + 1023) / 1024;
  const int chunks_x = (dx + kRaggedRows - 1) / kRaggedRows, chunks_h = (H + kRaggedRows - 1) / kRaggedRows;
  const int row_chunks = dW ? chunks_x + chunks_h + (db ? 1 : 0) : 1;
  PFG_KERNEL(outer_sum_ragged_kernel, dim3((unsigned)(col_chunks * row_chunks), (unsigned)B), dim3(256), 0, stream, p);
  return hipGetLastError();
}

}  // namespace pfg
