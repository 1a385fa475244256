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

// Condition and compaction of trip t in one workgroup, for lists of at most kPlace rows whose halting
// scores arrive in pieces (part[i * nparts + j], j < nparts, written by the step kernel of trip t - 1;
// all zero before the first trip).  Row m of the list: score = c0 + the pieces of iteration I[m] added
// in increasing j; the rest as in the two kernels above.
__global__ __launch_bounds__(kPlace) void while_select_one_kernel(const int32_t *I, const int32_t *meta, int t,
                                                                  const int32_t *seq_offsets, int total_tokens,
                                                                  const float *part, int nparts, float c0,
                                                                  int32_t *I_next, int32_t *meta_next,
                                                                  int32_t *steps, int32_t *trips) {
  constexpr int kWaves = kPlace / 64;
  __shared__ int s_wave[kWaves];
  const int l = min(meta[0], kPlace);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int f = 0, i = 0;
  if (tid < l) {
    i = I[tid];
    float s = 0.f;
    if (part) {
      const float *row = part + (int64_t)i * nparts;
      if ((nparts & 3) == 0 && (reinterpret_cast<uintptr_t>(part) & 15) == 0) {
        for (int j = 0; j < nparts; j += 4) {
          const f32x4 v = *reinterpret_cast<const f32x4 *>(row + j);
          s += v[0]; s += v[1]; s += v[2]; s += v[3];
        }
      } else {
        for (int j = 0; j < nparts; ++j) s += row[j];
      }
    }
    const int lo = seq_offsets[i], hi = min(seq_offsets[i + 1], total_tokens);
    const int len = (lo >= 0 && hi > lo) ? hi - lo : 0;
    f = (t < len && s + c0 <= 0.f) ? 1 : 0;
    if (!f) steps[i] = t;
  }
  const unsigned long long set = __ballot(f != 0);
  const int rank_in_wave = __popcll(set & ((1ull << lane) - 1ull));
  if (lane == 0) s_wave[wave] = __popcll(set);
  __syncthreads();
  int kept_before = 0, kept = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    kept += s_wave[w];
    if (w < wave) kept_before += s_wave[w];
  }
  if (f) I_next[kept_before + rank_in_wave] = i;
  if (tid == 0) {
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


// Per-iteration sums over the trips an iteration made (the same W acts in every trip, so an
// iteration's gradient is the sum of its trips' outer products; different iterations stay apart):
//   dW[b, 0:dx, :]      = sum_{t < T_b} x[r_b + t, :]^T     dz[r_b + t, :]
//   dW[b, dx:dx+H, :]   = sum_{1 <= t < T_b} h[r_b + t - 1, :]^T dz[r_b + t, :]      (h before trip 0 is zero)
//   db[b, :]            = sum_{t < T_b} dz[r_b + t, :]
// with r_b the iteration's first token row and T_b = steps[b] its trip count (both from device
// memory, cut to the iteration's token range).  Per iteration this is a product
// [x | h_prev]^T [dx + H, T_b] times dz [T_b, 4H] whose contraction length differs from iteration to
// iteration: it runs on the matrix cores (v_mfma_f32_32x32x2_f32, two trips per instruction).
//
// A wave takes 32 rows of one iteration's matrix and 32 NT columns; the four waves of a workgroup take
// four neighbouring row tiles of the same columns.  The columns are NT tiles of 32 x 32 whose columns
// interleave: lane l32 feeds columns base + NT l32 + e to tile e, so its cotangent values of a trip
// are one load of NT floats and register r of the NT tiles holds NT neighbouring columns of one output
// row, one store.  Three register sets of eight trips each are used in turn.  The result is written
// once, also when T_b = 0 (zeros).  The bias row is a plain sum in workgroups of its own.
//
// Measured on 1024 sequences of 1..100 tokens (41 148 trips, 1.61 GB out): stores alone (no trip)
// 0.29 ms, with the trips 0.57 ms; the time grows by the matrix-core time of the trips whose operands
// are fetched inside the loop, whatever the occupancy (NT = 2 at six waves per SIMD: 0.67 ms) and
// the depth of the ring.
constexpr int kRagGroup = 4;      // MFMA k-steps (of two trips) per register set

struct RaggedSumArgs {
  const float *x; int dx;
  const float *h_tok; int H;
  const float *dz_tok;           // [tokens, d_out], 16-byte aligned rows
  const int32_t *seq_offsets;    // [B + 1]
  const int32_t *steps;          // [B]
  int total_tokens;
  float *dW;                     // [B, dx + H, d_out] or nullptr
  float *db;                     // [B, d_out] or nullptr
  int d_out;                     // 4H
  int vec;                       // 16-byte stores allowed (alignment of dW, db)
  int mm_blocks;                 // workgroups per iteration that work on dW; the rest sum the bias row
};

template <int NT>   // column tiles per wave: 4 (16-byte operands), or 2 (8-byte operands, half the registers)
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(NT == 4 ? 3 : 6, NT == 4 ? 3 : 6)))
void outer_sum_ragged_kernel(const RaggedSumArgs p) {
  typedef float fv __attribute__((ext_vector_type(NT)));
  const int64_t b = blockIdx.y;
  const int lo = p.seq_offsets[b], hi = min(p.seq_offsets[b + 1], p.total_tokens);
  const int len = (lo >= 0 && hi > lo) ? hi - lo : 0;
  const int nt = max(0, min(p.steps[b], len));

  if ((int)blockIdx.x >= p.mm_blocks) {
    // ---- bias row: 1024 columns per workgroup, four per lane ----
    const int j = (((int)blockIdx.x - p.mm_blocks) * 256 + threadIdx.x) * 4;
    if (j >= p.d_out) return;
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    for (int t = 0; t < nt; ++t) s += *reinterpret_cast<const f32x4 *>(p.dz_tok + (int64_t)(lo + t) * p.d_out + j);
    float *o = p.db + b * (int64_t)p.d_out + j;
    if (p.vec) {
      *reinterpret_cast<f32x4 *>(o) = s;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = s[e];
    }
    return;
  }

  constexpr int WCOLS = 32 * NT;                           // columns of a wave's tile
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, half = lane >> 5;
  const int col_chunks = (p.d_out + WCOLS - 1) / WCOLS;
  const int cchunk = blockIdx.x % col_chunks, rtile = (blockIdx.x / col_chunks) * 4 + wave;
  const int R = p.dx + p.H;
  if (rtile * 32 >= R) return;                             // (no barrier follows)
  const int row = rtile * 32 + l32;                        // the row of [x | h_prev] this lane feeds
  const int col = cchunk * WCOLS + NT * l32;               // the first of this lane's NT columns
  const bool col_in = col < p.d_out;                       // d_out and col are multiples of NT
  // The operand values of trip t: this lane's row of [x_t | h_{t-1}] and its NT columns of dz_t; zero
  // for a trip the iteration did not make.  A lane takes the trips t0 + 2 s + half of a register set.
  // (Measured and not kept: loads without a branch on addresses clamped to the last trip, which lets
  // the compiler keep later sets in flight across the MFMAs -- the loads past the last trip that this
  // adds cost more than the overlap gains, 0.65 against 0.57 ms on 1024 sequences of 1..100 tokens.)
  const bool row_in = row < R, is_x = row < p.dx;
  const int t_first = is_x ? 0 : 1;                        // trip t pairs dz_t with h_{t-1}; h before trip 0 is zero
  const int64_t astride = is_x ? p.dx : p.H;
  // the two pointers stand at the lane's next trip, t_next
  const float *ap = (is_x ? p.x + (int64_t)lo * p.dx + row : p.h_tok + (int64_t)lo * p.H + (row - p.dx)) +
                    (half - t_first) * astride;
  const float *gp = p.dz_tok + ((int64_t)lo + half) * p.d_out + col;
  const int64_t a_step = 2 * astride, g_step = 2 * (int64_t)p.d_out;
  int t_next = half;
  const fv zero = {};
  auto fetch = [&](float (&a)[kRagGroup], fv (&g)[kRagGroup]) {
#pragma unroll
    for (int s = 0; s < kRagGroup; ++s) {
      a[s] = (row_in && t_next < nt && t_next >= t_first) ? *ap : 0.f;
      g[s] = (col_in && t_next < nt) ? *reinterpret_cast<const fv *>(gp) : zero;
      ap += a_step;
      gp += g_step;
      t_next += 2;
    }
  };

  f32x16 acc[NT];
#pragma unroll
  for (int e = 0; e < NT; ++e)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[e][r] = 0.f;
  // three register sets in turn: the operands of two sets are on their way while the MFMAs of one run
  float a_0[kRagGroup], a_1[kRagGroup], a_2[kRagGroup];
  fv g_0[kRagGroup], g_1[kRagGroup], g_2[kRagGroup];
  auto mma = [&](const float (&a)[kRagGroup], const fv (&g)[kRagGroup]) {
#pragma unroll
    for (int s = 0; s < kRagGroup; ++s)
#pragma unroll
      for (int e = 0; e < NT; ++e) acc[e] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[s], g[s][e], acc[e], 0, 0, 0);
  };
  constexpr int kTrips = 2 * kRagGroup;
  if (nt > 0) {
    fetch(a_0, g_0);
    fetch(a_1, g_1);
  }
#pragma unroll 1
  for (int t0 = 0; t0 < nt; t0 += 3 * kTrips) {
    fetch(a_2, g_2);
    mma(a_0, g_0);
    if (t0 + kTrips < nt) {
      fetch(a_0, g_0);
      mma(a_1, g_1);
      if (t0 + 2 * kTrips < nt) {
        fetch(a_1, g_1);
        mma(a_2, g_2);
      }
    }
  }

  if (!col_in) return;
  // register r of a tile is row 8 (r / 4) + 4 half + r % 4 of the tile, column l32
  float *out = p.dW + (b * (int64_t)R + rtile * 32) * p.d_out + col;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int i = 8 * (r >> 2) + 4 * half + (r & 3);
    if (rtile * 32 + i >= R) continue;
    fv v;
#pragma unroll
    for (int e = 0; e < NT; ++e) v[e] = acc[e][r];
    float *o = out + (int64_t)i * p.d_out;
    if (p.vec) {
      __builtin_nontemporal_store(v, reinterpret_cast<fv *>(o));
    } else {
#pragma unroll
      for (int e = 0; e < NT; ++e) o[e] = v[e];
    }
  }
}

// The same sums with the operands staged through LDS, for dx and H that are multiples of 4 (16-byte
// pieces never straddle the boundary between the x rows and the h rows): a workgroup takes 128 rows
// and 128 columns of one iteration's matrix and walks the trips in chunks of kLdsTrips.  All 256 threads
// fetch a chunk's operands -- [32 trips, 128 rows] of [x | h_prev] and [32 trips, 128 columns] of dz,
// eight 16-byte loads per thread, no value fetched twice -- while the MFMAs of the previous chunk
// run, and store them to LDS behind a barrier; wave w then feeds its 32 rows and the interleaved
// column tiles from LDS.  Against the register-fed kernel above: one exposure to memory latency per 32
// trips instead of one per 8, and 2.5 times fewer bytes requested.  Loads carry no branch (clamped
// to the iteration's last trip, last rows and last columns); what must be zero is zeroed on its way
// into LDS.
constexpr int kLdsTrips = 16;
constexpr int kLdsPieces = kLdsTrips / 8;    // 16-byte pieces of each operand a thread stages per chunk

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4))) void outer_sum_ragged_lds_kernel(const RaggedSumArgs p) {
  __shared__ __align__(16) float As[kLdsTrips][128];
  __shared__ __align__(16) float Gs[kLdsTrips][128];
  const int64_t b = blockIdx.y;
  const int lo = p.seq_offsets[b], hi = min(p.seq_offsets[b + 1], p.total_tokens);
  const int len = (lo >= 0 && hi > lo) ? hi - lo : 0;
  const int nt = max(0, min(p.steps[b], len));
  const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};

  if ((int)blockIdx.x >= p.mm_blocks) {
    // ---- bias row: 1024 columns per workgroup, four per lane ----
    const int j = (((int)blockIdx.x - p.mm_blocks) * 256 + threadIdx.x) * 4;
    if (j >= p.d_out) return;
    f32x4 s = zero4;
    for (int t = 0; t < nt; ++t) s += *reinterpret_cast<const f32x4 *>(p.dz_tok + (int64_t)(lo + t) * p.d_out + j);
    float *o = p.db + b * (int64_t)p.d_out + j;
    if (p.vec) {
      *reinterpret_cast<f32x4 *>(o) = s;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = s[e];
    }
    return;
  }

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, half = lane >> 5;
  const int col_chunks = (p.d_out + 127) / 128;
  const int cchunk = blockIdx.x % col_chunks, rgroup = blockIdx.x / col_chunks;
  const int R = p.dx + p.H;                                // a multiple of 4, like dx
  const int row0 = rgroup * 128, col0 = cchunk * 128;

  // staging: this thread's four pieces of a chunk are elements 4 part .. 4 part + 3 of the trips
  // tl0, tl0 + 8, ... of the chunk, for both operands
  const int part = tid & 31, tl0 = tid >> 5;
  const int ar = row0 + 4 * part, gcol = col0 + 4 * part;
  const bool a_in = ar < R, g_in = gcol < p.d_out;
  const int arc = min(ar, R - 4), gc = min(gcol, p.d_out - 4);
  const bool a_is_x = arc < p.dx;
  const int a_first = a_is_x ? 0 : 1;                      // trip t pairs dz_t with h_{t-1}; h before trip 0 is zero
  const int64_t astride = a_is_x ? p.dx : p.H;
  const float *abase = a_is_x ? p.x + (int64_t)lo * p.dx + arc : p.h_tok + (int64_t)lo * p.H + (arc - p.dx);
  const float *gbase = p.dz_tok + (int64_t)lo * p.d_out + gc;
  f32x4 ra[kLdsPieces], rg[kLdsPieces];
  auto fetch = [&](int t0) {                               // nt > 0
#pragma unroll
    for (int c = 0; c < kLdsPieces; ++c) {
      const int t = min(t0 + tl0 + 8 * c, nt - 1);
      ra[c] = *reinterpret_cast<const f32x4 *>(abase + max(t - a_first, 0) * astride);
      rg[c] = *reinterpret_cast<const f32x4 *>(gbase + (int64_t)t * p.d_out);
    }
  };
  auto stash = [&](int t0) {
#pragma unroll
    for (int c = 0; c < kLdsPieces; ++c) {
      const int tl = tl0 + 8 * c, t = t0 + tl;
      const bool live = t < nt;
      *reinterpret_cast<f32x4 *>(&As[tl][4 * part]) = (live && a_in && t >= a_first) ? ra[c] : zero4;
      *reinterpret_cast<f32x4 *>(&Gs[tl][4 * part]) = (live && g_in) ? rg[c] : zero4;
    }
  };

  f32x16 acc[4];
#pragma unroll
  for (int e = 0; e < 4; ++e)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[e][r] = 0.f;
  if (nt > 0) fetch(0);
#pragma unroll 1
  for (int t0 = 0; t0 < nt; t0 += kLdsTrips) {
    __syncthreads();                                       // the previous chunk has been read
    stash(t0);
    __syncthreads();
    if (t0 + kLdsTrips < nt) fetch(t0 + kLdsTrips);        // on its way while this chunk is multiplied
    const int pairs = min(kLdsTrips / 2, (nt - t0 + 1) / 2);
#pragma unroll 2
    for (int s = 0; s < pairs; ++s) {
      const float a = As[2 * s + half][32 * wave + l32];
      const f32x4 g = *reinterpret_cast<const f32x4 *>(&Gs[2 * s + half][4 * l32]);
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[e] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, g[e], acc[e], 0, 0, 0);
    }
  }

  const int rtile = rgroup * 4 + wave, col = col0 + 4 * l32;
  if (rtile * 32 >= R || col >= p.d_out) return;           // (no barrier follows)
  // register r of a tile is row 8 (r / 4) + 4 half + r % 4 of the tile, column l32
  float *out = p.dW + (b * (int64_t)R + rtile * 32) * p.d_out + col;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int i = 8 * (r >> 2) + 4 * half + (r & 3);
    if (rtile * 32 + i >= R) continue;
    const f32x4 v = {acc[0][r], acc[1][r], acc[2][r], acc[3][r]};
    float *o = out + (int64_t)i * p.d_out;
    if (p.vec) {
      __builtin_nontemporal_store(v, reinterpret_cast<f32x4 *>(o));
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = v[e];
    }
  }
}

// Squared norms of the per-example gradients through the while loop without the gradients.  With
// u_t = [x_t | h_{t-1}] and dz_t the rows of an iteration's trips,
//   |dW|^2 = |sum_t u_t^T dz_t|^2 = sum_{t, t'} (u_t . u_t') (dz_t . dz_t'),     |db|^2 = sum_{t, t'} dz_t . dz_t',
// i.e. the entries of the two T x T Gram matrices multiplied and added; |dWout|^2 = |h|^2 |gy|^2 and
// |dbout|^2 = |gy|^2 from the last state h and gy = d ell / d y.  One workgroup per iteration, at most
// kNormTrips trips.  The Gram matrices are products with themselves on the matrix cores: the rows of
// the operand (first dz, 4H long, then u, dx + H long) go through LDS in chunks of kNormK elements,
// fetched while the previous chunk is multiplied; only the 32 x 32 tiles on and above the diagonal that
// hold a trip are computed (each wave takes every fourth, at most three), an off-diagonal tile counts
// twice.  Rows past the last trip are staged as zeros.  Everything is added in a fixed order.
constexpr int kNormTrips = 128;
constexpr int kNormK = 64;
constexpr int kNormLd = kNormK + 1;      // row stride in floats: 32 consecutive rows of one column hit 32 banks
constexpr int kNormPieces = kNormTrips * (kNormK / 4) / 256;   // 16-byte pieces a thread stages per chunk

struct WhileNormArgs {
  const float *x; int dx;
  const float *h_tok; int H;
  const float *dz_tok;           // [tokens, 4H]
  const int32_t *seq_offsets;    // [B + 1]
  const int32_t *steps;          // [B]
  int total_tokens;
  const float *hfin;             // [B, H] last states
  const float *gy; int dy;       // [B, dy]
  float *sq;                     // [B, 4] or nullptr
  float *norm;                   // [B] or nullptr
  int vec;                       // x, h_tok 16-byte aligned, dx and H multiples of 4
};

__global__ __launch_bounds__(256) void while_grad_sqnorms_kernel(const WhileNormArgs p) {
  __shared__ float Zs[kNormTrips][kNormLd];
  __shared__ float red[2][4];
  __shared__ float tail[2];
  const int64_t b = blockIdx.x;
  const int lo = p.seq_offsets[b], hi = min(p.seq_offsets[b + 1], p.total_tokens);
  const int len = (lo >= 0 && hi > lo) ? hi - lo : 0;
  const int nt = max(0, min(min(p.steps[b], len), kNormTrips));
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, half = lane >> 5;
  const int G = 4 * p.H, KU = p.dx + p.H;
  const int nrt = (nt + 31) / 32;                          // row tiles that hold a trip
  const int ntiles = nrt * (nrt + 1) / 2;
  const int chunks_z = (G + kNormK - 1) / kNormK, chunks = chunks_z + (KU + kNormK - 1) / kNormK;

  // this wave's tiles (ti <= tj), numbered row by row over the upper triangle
  int ti[3], tj[3];
#pragma unroll
  for (int j = 0; j < 3; ++j) {
    int q = wave + 4 * j, r = 0;
    ti[j] = tj[j] = -1;
    if (q < ntiles) {
      while (q >= nrt - r) { q -= nrt - r; ++r; }
      ti[j] = r;
      tj[j] = r + q;
    }
  }

  // staging: piece c of this thread is elements 4 part .. 4 part + 3 of row tl0 + 16 c of the chunk
  const int part = tid & 15, tl0 = tid >> 4;
  f32x4 reg[kNormPieces];
  const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
  // element k of the operand row of trip t (clamped to a valid address; what must be zero is zeroed in stash)
  auto fetch = [&](int c) {                                // nt > 0
    const bool is_z = c < chunks_z;
    const int k = (is_z ? c : c - chunks_z) * kNormK + 4 * part;
    const int K = is_z ? G : KU;
#pragma unroll
    for (int i = 0; i < kNormPieces; ++i) {
      const int t = min(tl0 + 16 * i, nt - 1);
      if (p.vec || is_z) {
        const int kc = min(k, K - 4);                      // G, and with vec dx and H, are multiples of 4
        const float *src = is_z        ? p.dz_tok + (int64_t)(lo + t) * G + kc
                           : kc < p.dx ? p.x + (int64_t)(lo + t) * p.dx + kc
                                       : p.h_tok + (int64_t)(lo + max(t - 1, 0)) * p.H + (kc - p.dx);
        reg[i] = *reinterpret_cast<const f32x4 *>(src);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int ke = min(k + e, K - 1);
          reg[i][e] = ke < p.dx ? p.x[(int64_t)(lo + t) * p.dx + ke]
                                : p.h_tok[(int64_t)(lo + max(t - 1, 0)) * p.H + (ke - p.dx)];
        }
      }
    }
  };
  auto stash = [&](int c) {
    const bool is_z = c < chunks_z;
    const int k = (is_z ? c : c - chunks_z) * kNormK + 4 * part;
    const int K = is_z ? G : KU;
#pragma unroll
    for (int i = 0; i < kNormPieces; ++i) {
      const int t = tl0 + 16 * i;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        // u_0 has no recurrent part: h before trip 0 is zero
        const bool live = t < nt && k + e < K && (is_z || k + e < p.dx || t > 0);
        Zs[t][4 * part + e] = live ? reg[i][e] : 0.f;
      }
    }
  };

  f32x16 az[3], au[3];
#pragma unroll
  for (int j = 0; j < 3; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) az[j][r] = au[j][r] = 0.f;

  // one chunk of the operand's Gram matrix into acc (the tiles of this wave; a diagonal tile reads its
  // rows once)
  auto multiply = [&](f32x16 (&acc)[3]) {
#pragma unroll
    for (int j = 0; j < 3; ++j) {
      if (ti[j] < 0) continue;                             // wave-uniform
      const float *arow = &Zs[32 * ti[j] + l32][half], *brow = &Zs[32 * tj[j] + l32][half];
      if (ti[j] == tj[j]) {
#pragma unroll 8
        for (int s2 = 0; s2 < kNormK; s2 += 2) {
          const float v = arow[s2];
          acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(v, v, acc[j], 0, 0, 0);
        }
      } else {
#pragma unroll 8
        for (int s2 = 0; s2 < kNormK; s2 += 2)
          acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(arow[s2], brow[s2], acc[j], 0, 0, 0);
      }
    }
  };
  if (nt > 0) {
    fetch(0);
#pragma unroll 1
    for (int c = 0; c < chunks_z; ++c) {                   // dz dz^T
      __syncthreads();                                     // the previous chunk has been read
      stash(c);
      __syncthreads();
      fetch(c + 1);                                        // on its way while this chunk is multiplied (u follows dz)
      multiply(az);
    }
#pragma unroll 1
    for (int c = chunks_z; c < chunks; ++c) {              // u u^T
      __syncthreads();
      stash(c);
      __syncthreads();
      if (c + 1 < chunks) fetch(c + 1);
      multiply(au);
    }
  }

  // this wave's share: sum over its tiles of Gu o Gz and of Gz (off-diagonal tiles twice)
  float sw = 0.f, sb = 0.f;
#pragma unroll
  for (int j = 0; j < 3; ++j) {
    if (ti[j] < 0) continue;
    float tw = 0.f, tb = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      tw += az[j][r] * au[j][r];
      tb += az[j][r];
    }
    const float twice = ti[j] == tj[j] ? 1.f : 2.f;
    sw += twice * tw;
    sb += twice * tb;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    sw += __shfl_xor(sw, off, 64);
    sb += __shfl_xor(sb, off, 64);
  }
  if (lane == 0) {
    red[0][wave] = sw;
    red[1][wave] = sb;
  }
  // the readout: |h|^2 (wave 2) and |gy|^2 (wave 3)
  if (wave >= 2) {
    const float *v = wave == 2 ? p.hfin + b * (int64_t)p.H : p.gy + b * (int64_t)p.dy;
    const int n = wave == 2 ? p.H : p.dy;
    float s = 0.f;
    for (int k = lane; k < n; k += 64) s += v[k] * v[k];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if (lane == 0) tail[wave - 2] = s;
  }
  __syncthreads();
  if (tid == 0) {
    const float w2 = (red[0][0] + red[0][1]) + (red[0][2] + red[0][3]);
    const float b2 = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
    const float so = tail[0] * tail[1], sbo = tail[1];
    if (p.sq) {
      p.sq[4 * b] = w2; p.sq[4 * b + 1] = b2; p.sq[4 * b + 2] = so; p.sq[4 * b + 3] = sbo;
    }
    if (p.norm) p.norm[b] = sqrtf(w2 + b2 + so + sbo);
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
                               int32_t *steps, int32_t *trips, hipStream_t stream, const float *score_part,
                               int32_t score_ld) {
  static_assert(kWhileOneLaunchRows == kPlace, "the one-launch selection places its rows in one workgroup");
  if (B <= kPlace && (score_part || !w)) {
    PFG_KERNEL(while_select_one_kernel, dim3(1), dim3(kPlace), 0, stream, I, meta, t, seq_offsets, total_tokens,
               w ? score_part : nullptr, score_ld, c0, I_next, meta_next, steps, trips);
    return hipGetLastError();
  }
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

hipError_t launch_outer_sum_ragged(const float *x, int32_t dx, const float *h_tok, int32_t H, const float *dz_tok,
                                   const int32_t *seq_offsets, const int32_t *steps, int32_t total_tokens, int64_t B,
                                   float *dW, float *db, hipStream_t stream) {
  if (!dW && !db) return hipSuccess;
  if (B > 65535 || (reinterpret_cast<uintptr_t>(dz_tok) & 15)) return hipErrorInvalidConfiguration;
  RaggedSumArgs p{};
  p.x = x; p.dx = dx; p.h_tok = h_tok; p.H = H; p.dz_tok = dz_tok;
  p.seq_offsets = seq_offsets; p.steps = steps; p.total_tokens = total_tokens;
  p.dW = dW; p.db = db; p.d_out = 4 * H;
  p.vec = (((reinterpret_cast<uintptr_t>(dW) | reinterpret_cast<uintptr_t>(db)) & 15) == 0) ? 1 : 0;
  constexpr int NT = 4;
  const int col_chunks = (p.d_out + 32 * NT - 1) / (32 * NT), row_groups = (dx + H + 127) / 128;
  p.mm_blocks = dW ? col_chunks * row_groups : 0;
  const int bias_blocks = db ? (p.d_out + 1023) / 1024 : 0;
  const bool aligned = ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(h_tok)) & 15) == 0;
  if (dW && aligned && dx % 4 == 0 && H % 4 == 0)
    PFG_KERNEL(outer_sum_ragged_lds_kernel, dim3((unsigned)(p.mm_blocks + bias_blocks), (unsigned)B), dim3(256), 0,
               stream, p);
  else
    PFG_KERNEL(outer_sum_ragged_kernel<NT>, dim3((unsigned)(p.mm_blocks + bias_blocks), (unsigned)B), dim3(256), 0,
               stream, p);
  return hipGetLastError();
}

hipError_t launch_while_grad_sqnorms(const float *x, int32_t dx, const float *h_tok, int32_t H, const float *dz_tok,
                                     const int32_t *seq_offsets, const int32_t *steps, int32_t total_tokens,
                                     const float *hfin, const float *gy, int32_t dy, int64_t B, float *sq,
                                     float *norm, hipStream_t stream) {
  if (B <= 0 || (!sq && !norm)) return hipSuccess;
  if (B > 0x7fffffffLL || (reinterpret_cast<uintptr_t>(dz_tok) & 15)) return hipErrorInvalidValue;
  WhileNormArgs p{};
  p.x = x; p.dx = dx; p.h_tok = h_tok; p.H = H; p.dz_tok = dz_tok;
  p.seq_offsets = seq_offsets; p.steps = steps; p.total_tokens = total_tokens;
  p.hfin = hfin; p.gy = gy; p.dy = dy; p.sq = sq; p.norm = norm;
  p.vec = (((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(h_tok)) & 15) == 0 && dx % 4 == 0 &&
           H % 4 == 0) ? 1 : 0;
  PFG_KERNEL(while_grad_sqnorms_kernel, dim3((unsigned)B), dim3(256), 0, stream, p);
  return hipGetLastError();
}

}  // namespace pfg
