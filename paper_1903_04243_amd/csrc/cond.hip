// Kernels of the conditional inside a parallel-for (Section 3.6): the condition of every iteration
// is evaluated at once, then the flags are turned into the two index sets I_then and I_else, each in
// increasing order of the iteration index.  Both sets live in one array: the then-rows at the
// front, the else-rows behind them; `meta` tells the products that follow where each set starts and
// how long it is, so that the host never has to read a count back.
#include "common.h"

namespace pfg {

namespace {

constexpr int kGroup = 32;       // rows whose set flags are counted together
constexpr int kPlace = 1024;     // rows per workgroup of the placing kernel (a multiple of kGroup)

// flags[j] = (T[j, :] . w + c0 > 0); cnt[j / kGroup] = set flags in the group.  16 lanes share a row
// (each sums every 16th piece of the row, then a fixed xor tree joins the 16 partial sums); a
// workgroup of 256 threads takes one group of 32 rows in two passes.
__global__ __launch_bounds__(256) void cond_flags_kernel(const float *T, int64_t ldt, int n, int d,
                                                         const float *w, float c0, int32_t *flags,
                                                         int32_t *cnt) {
  __shared__ int s_cnt;
  if (threadIdx.x == 0) s_cnt = 0;
  __syncthreads();
  const int slot = threadIdx.x >> 4, l16 = threadIdx.x & 15;
  const bool vec = ((reinterpret_cast<uintptr_t>(T) | reinterpret_cast<uintptr_t>(w)) & 15) == 0 &&
                   ldt % 4 == 0 && d % 4 == 0;
  int mine = 0;
  for (int pass = 0; pass < kGroup / 16; ++pass) {
    const int row = blockIdx.x * kGroup + pass * 16 + slot;
    float s = 0.f;
    if (row < n) {
      const float *t = T + (int64_t)row * ldt;
      if (vec) {
        for (int k = 4 * l16; k < d; k += 64) {
          const f32x4 a = *reinterpret_cast<const f32x4 *>(t + k);
          const f32x4 b = *reinterpret_cast<const f32x4 *>(w + k);
          s += a[0] * b[0] + a[1] * b[1] + a[2] * b[2] + a[3] * b[3];
        }
      } else {
        for (int k = l16; k < d; k += 16) s += t[k] * w[k];
      }
    }
#pragma unroll
    for (int off = 8; off > 0; off >>= 1) s += __shfl_xor(s, off, 16);
    if (l16 == 0 && row < n) {
      const int f = (s + c0 > 0.f) ? 1 : 0;
      flags[row] = f;
      mine += f;
    }
  }
  if (l16 == 0 && mine) atomicAdd(&s_cnt, mine);      // integers: the order does not matter
  __syncthreads();
  if (threadIdx.x == 0) cnt[blockIdx.x] = s_cnt;
}

// blk[b] = sum of the kPlace / kGroup group counts of block b (the rows one placing workgroup takes).
// Only used for many rows, where every placing workgroup summing all group counts would cost more
// than this extra launch.
__global__ __launch_bounds__(256) void cond_block_counts_kernel(const int32_t *cnt, int ngroups, int nblocks,
                                                                int32_t *blk) {
  constexpr int kPer = kPlace / kGroup;
  const int b = blockIdx.x * 256 + threadIdx.x;
  if (b >= nblocks) return;
  int s = 0;
  for (int g = b * kPer; g < min((b + 1) * kPer, ngroups); ++g) s += cnt[g];
  blk[b] = s;
}

// Row j with a set flag goes to rows[(set flags before j)], a row with a clear flag to
// rows[n_then + (clear flags before j)].  A workgroup places kPlace consecutive rows: it sums the
// counts in front of its rows (and all of them, for n_then) -- group counts, or block counts when
// blk is given --, ranks its own rows with a ballot per wave, and writes.
// meta = {n_then, 0, n_else, n_then}: count and offset of each set.
__global__ __launch_bounds__(kPlace) void cond_place_kernel(const int32_t *flags, const int32_t *cnt,
                                                            const int32_t *blk, int n, int32_t *rows,
                                                            int32_t *meta, int32_t *cond_out,
                                                            int32_t *counts_out) {
  constexpr int kWaves = kPlace / 64;
  __shared__ int s_before[kWaves], s_total[kWaves], s_wave[kWaves];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // counts to add up: one per block of kPlace rows, or one per group of kGroup rows
  const int32_t *c = blk ? blk : cnt;
  const int per = blk ? kPlace : kGroup;
  const int ncounts = (n + per - 1) / per;
  const int first = blockIdx.x * (kPlace / per);          // first count that belongs to this workgroup
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
  const int j = blockIdx.x * kPlace + tid;
  const int f = (j < n) ? flags[j] : 0;
  const unsigned long long set = __ballot(f != 0);
  const int rank_in_wave = __popcll(set & ((1ull << lane) - 1ull));
  if (lane == 0) {
    s_before[wave] = before;
    s_total[wave] = total;
    s_wave[wave] = __popcll(set);
  }
  __syncthreads();
  int then_before = 0, n_then = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    then_before += s_before[w];
    n_then += s_total[w];
    if (w < wave) then_before += s_wave[w];
  }
  if (j < n) {
    const int r = then_before + rank_in_wave;            // set flags in front of row j
    rows[f ? r : n_then + (j - r)] = j;
    if (cond_out) cond_out[j] = f;
  }
  if (blockIdx.x == 0 && tid == 0) {
    meta[0] = n_then;
    meta[1] = 0;
    meta[2] = n - n_then;
    meta[3] = n_then;
    if (counts_out) {
      counts_out[0] = n_then;
      counts_out[1] = n - n_then;
    }
  }
}

// out[0 .. n) = value (int32)
__global__ __launch_bounds__(256) void fill_int_kernel(int32_t *out, int n, int32_t value) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) out[i] = value;
}

// counts_out = {n or 0, 0 or n} for a loop-invariant condition
__global__ void invariant_counts_kernel(int32_t *counts_out, int n, int flag) {
  if (threadIdx.x == 0) {
    counts_out[0] = flag ? n : 0;
    counts_out[1] = flag ? 0 : n;
  }
}

// rows[m] = m, meta = the two descriptors of a loop-invariant condition: every row in one set
__global__ __launch_bounds__(256) void cond_identity_list_kernel(int32_t *rows, int32_t *meta, int n, int flag) {
  const int m = blockIdx.x * 256 + threadIdx.x;
  if (m < n) rows[m] = m;
  if (m == 0) {
    meta[0] = flag ? n : 0;
    meta[1] = 0;
    meta[2] = flag ? 0 : n;
    meta[3] = flag ? n : 0;
  }
}

// out[rows[m], :] = position m of the list lies in the set {sub[1] .. sub[1] + sub[0] - 1} ?
//                   src[gather ? rows[m] : m - sub[1], :] : 0          for m < n, d columns
__global__ __launch_bounds__(256) void cond_scatter_rows_kernel(const float *src, int64_t ld_src, int gather,
                                                                const int32_t *rows, const int32_t *sub, int n,
                                                                int d, float *out, int64_t ld_out) {
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= (int64_t)n * d) return;
  const int m = (int)(e / d), j = (int)(e - (int64_t)m * d);
  const int p = m - sub[1];
  const int row = rows[m];
  const bool live = p >= 0 && p < sub[0];
  out[(int64_t)row * ld_out + j] = live ? src[(int64_t)(gather ? row : p) * ld_src + j] : 0.f;
}

}  // namespace

hipError_t launch_cond_identity_list(int32_t *rows, int32_t *meta, int32_t n, int32_t flag, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  PFG_KERNEL(cond_identity_list_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, rows, meta, n, flag);
  return hipGetLastError();
}

hipError_t launch_cond_scatter_rows(const float *src, int64_t ld_src, int32_t gather, const int32_t *rows,
                                    const int32_t *sub, int32_t n, int32_t d, float *out, int64_t ld_out,
                                    hipStream_t stream) {
  if (n <= 0 || d <= 0) return hipSuccess;
  const int64_t total = (int64_t)n * d;
  PFG_KERNEL(cond_scatter_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, src, ld_src,
             gather, rows, sub, n, d, out, ld_out);
  return hipGetLastError();
}

// counts kept in `cnt`: one per group of kGroup rows, followed by one per block of kPlace rows
int64_t cond_count_groups(int64_t n) { return (n + kGroup - 1) / kGroup + (n + kPlace - 1) / kPlace; }

hipError_t launch_cond_partition(const float *T, int64_t ldt, int32_t n, int32_t d, const float *w,
                                 float c0, int32_t *flags, int32_t *cnt, int32_t *rows, int32_t *meta,
                                 int32_t *cond_out, int32_t *counts_out, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  const int ngroups = (n + kGroup - 1) / kGroup, nblocks = (n + kPlace - 1) / kPlace;
  PFG_KERNEL(cond_flags_kernel, dim3((unsigned)ngroups), dim3(256), 0, stream, T, ldt, n, d, w, c0, flags, cnt);
  // beyond 64 Ki rows (2048 group counts) the placing workgroups add up block counts instead
  int32_t *blk = nullptr;
  if (n > (1 << 16)) {
    blk = cnt + ngroups;
    PFG_KERNEL(cond_block_counts_kernel, dim3((unsigned)((nblocks + 255) / 256)), dim3(256), 0, stream, cnt,
               ngroups, nblocks, blk);
  }
  PFG_KERNEL(cond_place_kernel, dim3((unsigned)nblocks), dim3(kPlace), 0, stream, flags, cnt, blk, n, rows, meta,
             cond_out, counts_out);
  return hipGetLastError();
}

hipError_t launch_cond_invariant(int32_t n, int32_t flag, int32_t *cond_out, int32_t *counts_out,
                                 hipStream_t stream) {
  if (cond_out && n > 0)
    PFG_KERNEL(fill_int_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, cond_out, n,
               flag ? 1 : 0);
  if (counts_out) PFG_KERNEL(invariant_counts_kernel, dim3(1), dim3(64), 0, stream, counts_out, n, flag);
  return hipGetLastError();
}

}  // namespace pfg
