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

}  // namespace pfg
