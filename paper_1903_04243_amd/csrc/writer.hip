// Per-instance outer-product writer:  out[m, i, j] = a[m / S, i] * g[m, j].
//
// Section 3.4: a matmul whose operands are BOTH loop-variant becomes a batch_matmul over the
// stacked iterations.  The weight gradient of one iteration is the [d_in, 1] x [1, d_out] product
// of the layer input and the cotangent row, a contraction of length one, so the "batched matmul"
// degenerates into one multiply per output value and the kernel is bound by how fast HBM absorbs
// the stacked [M, d_in, d_out] result.  It is therefore a pure streaming writer: every lane holds
// four consecutive g values in registers, multiplies them by one a value per row and issues one
// 16-byte non-temporal store per row; consecutive lanes cover consecutive 16-byte pieces of a row
// and a workgroup walks a contiguous run of rows of one iteration m.  The outer products of all
// layers of a call share one launch.
#include <vector>

#include "common.h"
#include "host.h"

namespace pfg {

namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ float load_a(const void *a, int a_bf16, int64_t idx) {
  if (a_bf16) return (float)static_cast<const __bf16 *>(a)[idx];
  return static_cast<const float *>(a)[idx];
}

// One unit of work of the launch: a stacked outer product and how one iteration m of it is cut
// into workgroups.
struct OuterJob {
  OuterArgs o;
  int32_t vec;              // 1: 16-byte stores (d_out % 4 == 0, out 16-byte aligned); 0: scalar
  int32_t V;                // vec: d_out / 4 vector columns
  int32_t slabs;            // vec: column slabs of up to THREADS vectors
  int32_t chunks;           // row chunks (vec) or flat element chunks (scalar) per iteration m
  int32_t per_chunk;        // rows (vec) or elements (scalar) per chunk
  uint32_t x_begin;         // first blockIdx.x of this job
};

constexpr int kMaxJobs = 8;
struct OuterBatch {
  OuterJob job[kMaxJobs];
  int32_t n;
  int64_t M;                // iterations, the same for every job of a launch
};

// The index arithmetic below is kept to 32-bit, wave-uniform operations (and none at all in the
// common one-slab case): a workgroup issues only a few stores per lane, so a long prologue would
// cost more than the stores.

// d_out % 4 == 0, out 16-byte aligned.  V = d_out / 4 vector columns.
// Workgroup = (m, column slab of up to THREADS vectors, chunk of rows).  When V < THREADS a pass
// covers THREADS / V rows at once.
// m: the slice of `out` that is written; ma, mg: the rows of a and g it is the product of; live:
// false writes zeros instead (a row of a device-side list that lies outside the job's set).
template <int THREADS>
__device__ __forceinline__ void outer_vec4(const OuterJob &jb, uint32_t x, int64_t m, int64_t ma, int64_t mg,
                                           bool live) {
  const OuterArgs &o = jb.o;
  const int V = jb.V;
  uint32_t chunk = x, slab = 0;
  if (jb.slabs > 1) {
    // consecutive workgroups take consecutive slabs of the same rows, so that the launch as a
    // whole writes memory in address order (rows walked first put neighbouring workgroups a power
    // of two apart: 65 % instead of 80 % of the HBM peak on 4096-wide rows)
    slab = x % (uint32_t)jb.slabs;
    chunk = x / (uint32_t)jb.slabs;
  }

  int vc, r0, rstep;
  if (V >= THREADS) {
    vc = slab * THREADS + threadIdx.x;
    r0 = 0;
    rstep = 1;
  } else {
    rstep = THREADS / V;
    r0 = threadIdx.x / V;
    vc = threadIdx.x - r0 * V;
    if (r0 >= rstep) return;           // lanes beyond the last whole row of a pass idle
  }
  if (vc >= V) return;

  const int i_begin = chunk * jb.per_chunk;
  const int i_end = min(i_begin + jb.per_chunk, o.d_in);
  f32x4 *obase = reinterpret_cast<f32x4 *>(o.out + m * (int64_t)o.d_in * o.d_out) + vc;
  if (!live) {
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    for (int i = i_begin + r0; i < i_end; i += rstep) __builtin_nontemporal_store(zero, obase + (int64_t)i * V);
    return;
  }

  const float *grow = o.g + mg * o.ldg + 4 * vc;
  f32x4 gv;
  if (((reinterpret_cast<uintptr_t>(o.g) & 15) == 0) && ((o.ldg & 3) == 0)) {
    gv = *reinterpret_cast<const f32x4 *>(grow);
  } else {
    gv[0] = grow[0]; gv[1] = grow[1]; gv[2] = grow[2]; gv[3] = grow[3];
  }

  const int64_t abase = ma * o.lda;
  for (int i = i_begin + r0; i < i_end; i += rstep) {
    const float av = load_a(o.a, o.a_bf16, abase + i);
    __builtin_nontemporal_store(gv * av, obase + (int64_t)i * V);
  }
}

// Any d_out, any alignment: one thread per output value of a flattened [d_in * d_out] iteration.
template <int THREADS>
__device__ __forceinline__ void outer_flat(const OuterJob &jb, uint32_t chunk, int64_t m, int64_t ma, int64_t mg,
                                           bool live) {
  const OuterArgs &o = jb.o;
  const int64_t per_m = (int64_t)o.d_in * o.d_out;
  const int64_t e_begin = (int64_t)chunk * jb.per_chunk;
  const int64_t e_end = min(e_begin + jb.per_chunk, per_m);
  const int64_t abase = ma * o.lda;
  const float *grow = o.g + mg * o.ldg;
  float *obase = o.out + m * per_m;
  if (!live) {
    for (int64_t e = e_begin + threadIdx.x; e < e_end; e += THREADS) obase[e] = 0.f;
    return;
  }
  for (int64_t e = e_begin + threadIdx.x; e < e_end; e += THREADS) {
    const uint32_t i = (uint32_t)e / (uint32_t)o.d_out;     // per_m < 2^31 is checked by the host
    const uint32_t j = (uint32_t)e - i * (uint32_t)o.d_out;
    obase[e] = load_a(o.a, o.a_bf16, abase + i) * grow[j];
  }
}

// All outer products of one call go out in a single launch:
// blockIdx.x selects the job and the piece of one iteration, blockIdx.y/z the iteration m.  The
// ramp-up and tail of a streaming kernel are then paid once and small layers fill in between
// large ones.
// SUBSET: the jobs' iterations are the entries of a device-side list (OuterArgs::sub, sub_rows):
// grid index m is a position in the list, the slice written is that of row sub_rows[m], and
// positions outside the job's set {offset .. offset + count - 1} get zeros.  Kept in an
// instantiation of its own: the plain kernel carries none of these loads.
template <int THREADS, bool SUBSET>
__global__ __launch_bounds__(THREADS) void outer_product_kernel(const OuterBatch batch) {
  const int64_t m = (int64_t)blockIdx.z * gridDim.y + blockIdx.y;
  if (m >= batch.M) return;
  const uint32_t x = blockIdx.x;
  int j = 0;
#pragma unroll
  for (int t = 1; t < kMaxJobs; ++t)
    if (t < batch.n && x >= batch.job[t].x_begin) j = t;
  const OuterJob &jb = batch.job[j];
  int64_t mo = m, ma, mg = m;
  bool live = true;
  if (SUBSET) {
    const OuterArgs &o = jb.o;
    const int count = o.sub[0], off = o.sub[1];
    const int64_t p = m - off;                   // position inside the job's set
    live = p >= 0 && p < count;
    mo = o.sub_rows[m];
    ma = o.a_gather ? mo : p;
    mg = o.g_gather ? mo : p;
  } else {
    ma = jb.o.S == 1 ? m : (int64_t)((uint32_t)m / (uint32_t)jb.o.S);
  }
  if (jb.vec)
    outer_vec4<THREADS>(jb, x - jb.x_begin, mo, ma, mg, live);
  else
    outer_flat<THREADS>(jb, x - jb.x_begin, mo, ma, mg, live);
}

// Wide rows of a large output (d_out >= 1024, at least kWideBytes in all): a kernel of its own with
// next to no prologue.  A workgroup is one 4 KiB slab of one row -- grid = (slabs, rows, iterations),
// so no index is ever divided -- and every lane issues a single 16-byte store.  Measured on plain
// fills and on this product (17 GB, rows of 16 KiB): 4 KiB per workgroup streams at 6.6 to 7.0 TB/s,
// 8 KiB at 6.1 to 6.4, 16 KiB at 5.8 to 6.2; the general kernel above cannot go below 8 KiB because
// its prologue (job table, chunk arithmetic) then costs more than its stores.
constexpr int64_t kWideBytes = (int64_t)128 << 20;

template <bool A_BF16, bool SEEDS>
__global__ __launch_bounds__(kThreads) void outer_wide_kernel(const void *__restrict__ a, int64_t lda,
                                                              const float *__restrict__ g, int64_t ldg,
                                                              float *__restrict__ out, int d_in, int V,
                                                              int S) {
  const int vc = blockIdx.x * kThreads + threadIdx.x;
  const uint32_t i = blockIdx.y;
  const int64_t m = blockIdx.z;
  if (vc >= V) return;
  const f32x4 gv = *reinterpret_cast<const f32x4 *>(g + m * ldg + 4 * vc);
  const int64_t arow = (SEEDS ? (int64_t)((uint32_t)m / (uint32_t)S) : m) * lda + i;
  const float av = A_BF16 ? (float)static_cast<const __bf16 *>(a)[arow] : static_cast<const float *>(a)[arow];
  f32x4 *o = reinterpret_cast<f32x4 *>(out) + (m * d_in + i) * (int64_t)V + vc;
  __builtin_nontemporal_store(gv * av, o);
}

// The same for iterations taken from a device-side list (float32 a, no seed axis): grid index z is a
// position in the list, the slice written is that of row sub_rows[z]; a position outside the job's set
// {offset .. offset + count - 1} gets zeros.  The list entry and the two descriptor words are
// wave-uniform loads.
__global__ __launch_bounds__(kThreads) void outer_wide_subset_kernel(const float *__restrict__ a, int64_t lda,
                                                                     const float *__restrict__ g, int64_t ldg,
                                                                     float *__restrict__ out, int d_in, int V,
                                                                     const int32_t *__restrict__ sub,
                                                                     const int32_t *__restrict__ sub_rows,
                                                                     int a_gather, int g_gather) {
  const int vc = blockIdx.x * kThreads + threadIdx.x;
  const uint32_t i = blockIdx.y;
  const int m = blockIdx.z;
  if (vc >= V) return;
  const int p = m - sub[1];
  const int64_t mo = sub_rows[m];
  f32x4 v = {0.f, 0.f, 0.f, 0.f};
  if (p >= 0 && p < sub[0]) {
    const int64_t ma = a_gather ? mo : p, mg = g_gather ? mo : p;
    v = *reinterpret_cast<const f32x4 *>(g + mg * ldg + 4 * vc) * a[ma * lda + i];
  }
  __builtin_nontemporal_store(v, reinterpret_cast<f32x4 *>(out) + (mo * d_in + i) * (int64_t)V + vc);
}

// Narrow rows (d_out = 256 or 512 floats) of a very large output: the same one-store-per-lane shape, a
// workgroup = one 4 KiB slab = ROWS whole rows of one iteration's matrix.
template <bool A_BF16, int ROWS>
__global__ __launch_bounds__(kThreads) void outer_wide_rows_kernel(const void *__restrict__ a, int64_t lda,
                                                                   const float *__restrict__ g, int64_t ldg,
                                                                   float *__restrict__ out, int d_in) {
  constexpr int VL = kThreads / ROWS;            // lanes per row = d_out / 4
  const int vc = threadIdx.x % VL;
  const uint32_t i = blockIdx.x * ROWS + threadIdx.x / VL;
  const int64_t m = blockIdx.y;
  if (i >= (uint32_t)d_in) return;
  const f32x4 gv = *reinterpret_cast<const f32x4 *>(g + m * ldg + 4 * vc);
  const int64_t arow = m * lda + i;
  const float av = A_BF16 ? (float)static_cast<const __bf16 *>(a)[arow] : static_cast<const float *>(a)[arow];
  f32x4 *o = reinterpret_cast<f32x4 *>(out) + (m * d_in + i) * (int64_t)VL + vc;
  __builtin_nontemporal_store(gv * av, o);
}

// From half a GiB per layer on (measured on the 784-512-512-10 network: at batch 256, 411 MB in the
// first layer, the general kernel with all layers in one launch is still level or better, 0.134 against
// 0.137 ms; at batch 512 0.263 -> 0.248 ms, at 2048 0.949 -> 0.859 ms = 7.2 TB/s in these launches)
constexpr int64_t kNarrowBytes = (int64_t)512 << 20;

// 0: no; 2 or 4: rows per workgroup
int wide_rows_applies(const OuterArgs &o) {
  if (o.sub || o.S != 1 || (o.d_out != 256 && o.d_out != 512) || o.M > 65535) return 0;
  if ((reinterpret_cast<uintptr_t>(o.out) | reinterpret_cast<uintptr_t>(o.g)) & 15) return 0;
  if (o.ldg & 3) return 0;
  if (o.M * (int64_t)o.d_in * o.d_out * 4 < kNarrowBytes) return 0;
  return 1024 / o.d_out;
}

hipError_t launch_wide_rows(const OuterArgs &o, int rows, hipStream_t stream) {
  const dim3 grid((unsigned)((o.d_in + rows - 1) / rows), (unsigned)o.M);
#define PFG_WIDE_ROWS(BF, R)                                                                                  \
  PFG_KERNEL((outer_wide_rows_kernel<BF, R>), grid, dim3(kThreads), 0, stream, o.a, o.lda, o.g, o.ldg, o.out, \
             o.d_in)
  if (o.a_bf16) {
    if (rows == 2) PFG_WIDE_ROWS(true, 2); else PFG_WIDE_ROWS(true, 4);
  } else {
    if (rows == 2) PFG_WIDE_ROWS(false, 2); else PFG_WIDE_ROWS(false, 4);
  }
#undef PFG_WIDE_ROWS
  return hipGetLastError();
}

bool wide_applies(const OuterArgs &o) {
  if (o.sub && (!o.sub_rows || o.a_bf16 || o.S != 1)) return false;
  if (o.d_out % 4 || o.d_out < 4 * kThreads || o.M > 65535 || o.d_in > 65535) return false;
  if ((reinterpret_cast<uintptr_t>(o.out) | reinterpret_cast<uintptr_t>(o.g)) & 15) return false;
  if (o.ldg & 3) return false;
  return o.M * (int64_t)o.d_in * o.d_out * 4 >= kWideBytes;
}

hipError_t launch_wide(const OuterArgs &o, hipStream_t stream) {
  const int V = o.d_out / 4;
  const dim3 grid((unsigned)((V + kThreads - 1) / kThreads), (unsigned)o.d_in, (unsigned)o.M);
  if (o.sub) {
    PFG_KERNEL(outer_wide_subset_kernel, grid, dim3(kThreads), 0, stream, static_cast<const float *>(o.a), o.lda, o.g,
               o.ldg, o.out, o.d_in, V, o.sub, o.sub_rows, o.a_gather, o.g_gather);
    return hipGetLastError();
  }
#define PFG_WIDE(BF, SD)                                                                              \
  PFG_KERNEL((outer_wide_kernel<BF, SD>), grid, dim3(kThreads), 0, stream, o.a, o.lda, o.g, o.ldg, o.out, \
             o.d_in, V, o.S)
  if (o.a_bf16) {
    if (o.S == 1) PFG_WIDE(true, false); else PFG_WIDE(true, true);
  } else {
    if (o.S == 1) PFG_WIDE(false, false); else PFG_WIDE(false, true);
  }
#undef PFG_WIDE
  return hipGetLastError();
}

// Cuts one iteration of an outer product into workgroups; returns how many.
int64_t plan_job(const OuterArgs &o, OuterJob &jb, int64_t target) {
  constexpr int threads = kThreads;
  jb.o = o;
  jb.vec = (o.d_out % 4 == 0) && ((reinterpret_cast<uintptr_t>(o.out) & 15) == 0);
  if (jb.vec) {
    const int V = o.d_out / 4;
    jb.V = V;
    jb.slabs = V >= threads ? (V + threads - 1) / threads : 1;
    const int rows_per_pass = V >= threads ? 1 : threads / V;
    const int64_t pass_bytes = (int64_t)rows_per_pass * (V >= threads ? threads : V) * 16;
    int passes = (int)((target + pass_bytes - 1) / pass_bytes);
    if (passes < 1) passes = 1;
    int rows_per_chunk = passes * rows_per_pass;
    if (rows_per_chunk > o.d_in)
      rows_per_chunk = ((o.d_in + rows_per_pass - 1) / rows_per_pass) * rows_per_pass;
    jb.per_chunk = rows_per_chunk;
    jb.chunks = (o.d_in + rows_per_chunk - 1) / rows_per_chunk;
    return (int64_t)jb.slabs * jb.chunks;
  }
  const int64_t per_m = (int64_t)o.d_in * o.d_out;
  jb.V = 0;
  jb.slabs = 1;
  jb.per_chunk = 4096;
  jb.chunks = (int)((per_m + jb.per_chunk - 1) / jb.per_chunk);
  return jb.chunks;
}

// One launch per group of jobs with the same iteration count (normally all of them).
hipError_t launch_class(const OuterArgs *jobs, int n, int64_t M, bool subset, int64_t target, hipStream_t stream) {
  int at = 0;
  while (at < n) {
    OuterBatch batch{};
    batch.M = M;
    int64_t xs = 0;
    while (at < n && batch.n < kMaxJobs) {
      const OuterArgs &o = jobs[at++];
      if (o.M != M || (o.sub != nullptr) != subset || o.d_in <= 0 || o.d_out <= 0) continue;
      OuterJob &jb = batch.job[batch.n];
      const int64_t nx = plan_job(o, jb, target);
      if (xs + nx > 0x7fffffffLL) {
        if (batch.n == 0) return hipErrorInvalidConfiguration;   // one job alone is too large
        --at;                                                    // start a new launch with it
        break;
      }
      jb.x_begin = (uint32_t)xs;
      xs += nx;
      ++batch.n;
    }
    if (batch.n == 0) continue;
    const unsigned gy = (unsigned)(M < 65535 ? M : 65535);
    const unsigned gz = (unsigned)((M + gy - 1) / gy);
    if (gz > 65535) return hipErrorInvalidConfiguration;
    const dim3 grid((unsigned)xs, gy, gz);
    if (subset)
      PFG_KERNEL((outer_product_kernel<kThreads, true>), grid, dim3(kThreads), 0, stream, batch);
    else
      PFG_KERNEL((outer_product_kernel<kThreads, false>), grid, dim3(kThreads), 0, stream, batch);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

// The plainest write stream there is, for measuring what HBM absorbs: out[0 .. n) = value with PER
// 16-byte non-temporal stores per lane (a workgroup covers PER * 4 KiB of consecutive addresses,
// lane t writing pieces t, t + 256, ...), workgroups in address order.  n is a multiple of 4, out
// 16-byte aligned.
template <int PER>
__global__ __launch_bounds__(kThreads) void fill_reference_kernel(float *out, int64_t nvec, float value) {
  const int64_t base = ((int64_t)blockIdx.y * gridDim.x + blockIdx.x) * (PER * kThreads) + threadIdx.x;
  const f32x4 v = {value, value, value, value};
  f32x4 *o = reinterpret_cast<f32x4 *>(out);
#pragma unroll
  for (int u = 0; u < PER; ++u)
    if (base + u * kThreads < nvec) __builtin_nontemporal_store(v, o + base + u * kThreads);
}

}  // namespace

hipError_t launch_fill_reference(float *out, int64_t n, float value, int stores_per_lane, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  if ((n & 3) || (reinterpret_cast<uintptr_t>(out) & 15)) return hipErrorInvalidValue;
  const int64_t nvec = n / 4;
  const int64_t per = (int64_t)stores_per_lane * kThreads;
  const int64_t groups = (nvec + per - 1) / per;
  const unsigned gx = (unsigned)(groups < 65535 ? groups : 65535);
  const int64_t gy = (groups + gx - 1) / gx;
  if (gy > 65535) return hipErrorInvalidConfiguration;
  const dim3 grid(gx, (unsigned)gy);
  switch (stores_per_lane) {
    case 1: PFG_KERNEL(fill_reference_kernel<1>, grid, dim3(kThreads), 0, stream, out, nvec, value); break;
    case 2: PFG_KERNEL(fill_reference_kernel<2>, grid, dim3(kThreads), 0, stream, out, nvec, value); break;
    case 4: PFG_KERNEL(fill_reference_kernel<4>, grid, dim3(kThreads), 0, stream, out, nvec, value); break;
    case 8: PFG_KERNEL(fill_reference_kernel<8>, grid, dim3(kThreads), 0, stream, out, nvec, value); break;
    case 16: PFG_KERNEL(fill_reference_kernel<16>, grid, dim3(kThreads), 0, stream, out, nvec, value); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_outer(const OuterArgs *jobs, int n, hipStream_t stream) {
  // Workgroup size and store kind, from sweeps of this kernel on MI355X (a purely sequential fill
  // with 16-byte stores reaches 6.0 to 6.7 TB/s there, hipMemset 6.0 to 6.5).  Many small
  // independent workgroups do best: 8 KiB each (two stores per lane), non-temporal stores, for
  // every shape and size tried (85 MB to 34 GB; rows of 1 KiB to 16 KiB).  Non-temporal stores
  // also leave the caches to the kernels that follow (the conv net's step is 5 % shorter although
  // its writer is not).  16 KiB per workgroup: 5 to 15 % slower; 4 KiB (one store per lane): the
  // index prologue dominates.
  const int64_t target = 8192;
  // large outputs with wide rows leave in launches of their own (see outer_wide_kernel)
  constexpr int kInline = 32;                  // no host allocation for the usual few jobs
  OuterArgs rest_inline[kInline];
  std::vector<OuterArgs> rest_heap;
  if (n > kInline) rest_heap.resize(n);
  OuterArgs *rest = n > kInline ? rest_heap.data() : rest_inline;
  int nrest = 0;
  for (int i = 0; i < n; ++i) {
    if (jobs[i].M > 0 && jobs[i].d_in > 0 && wide_applies(jobs[i])) {
      set_timing_family("outer_product_wide");
      hipError_t e = launch_wide(jobs[i], stream);
      if (e != hipSuccess) return e;
    } else if (jobs[i].M > 0 && jobs[i].d_in > 0 && wide_rows_applies(jobs[i])) {
      set_timing_family("outer_product_wide");
      hipError_t e = launch_wide_rows(jobs[i], wide_rows_applies(jobs[i]), stream);
      if (e != hipSuccess) return e;
    } else {
      rest[nrest++] = jobs[i];
    }
  }
  set_timing_family("outer_product");
  jobs = rest;
  n = nrest;
  for (int i = 0; i < n; ++i) {
    if (jobs[i].M <= 0) continue;
    if ((int64_t)jobs[i].d_in * jobs[i].d_out > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    const bool subset = jobs[i].sub != nullptr;
    if (subset && (!jobs[i].sub_rows || jobs[i].S != 1)) return hipErrorInvalidValue;
    bool seen = false;
    for (int k = 0; k < i; ++k) seen = seen || (jobs[k].M == jobs[i].M && (jobs[k].sub != nullptr) == subset);
    if (seen) continue;
    hipError_t e = launch_class(jobs, n, jobs[i].M, subset, target, stream);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace pfg
