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
#include "common.h"

namespace pfg {

namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ float load_a(const void *a, int a_bf16, int64_t idx) {
  if (a_bf16) return (float)static_cast<const __bf16 *>(a)[idx];
  return static_cast<const float *>(a)[idx];
}

// One unit of work of the launch: a stacked outer product and how it is cut into workgroups.
struct OuterJob {
  OuterArgs o;
  int32_t vec;              // 1: 16-byte stores (d_out % 4 == 0, out 16-byte aligned); 0: scalar
  int32_t V;                // vec: d_out / 4 vector columns
  int32_t slabs;            // vec: column slabs of up to 256 vectors
  int32_t chunks;           // row chunks (vec) or flat element chunks (scalar) per iteration m
  int32_t per_chunk;        // rows (vec) or elements (scalar) per chunk
  int64_t block_begin;      // first workgroup id of this job inside the launch
};

constexpr int kMaxJobs = 8;
struct OuterBatch {
  OuterJob job[kMaxJobs];
  int32_t n;
};

// d_out % 4 == 0, out 16-byte aligned.  V = d_out / 4 vector columns.
// Workgroup = (m, column slab of up to 256 vectors, chunk of rows).  When V < 256 a pass covers
// 256 / V rows at once.
__device__ __forceinline__ void outer_vec4(const OuterJob &jb, int64_t bid) {
  const OuterArgs &o = jb.o;
  const int V = jb.V;
  const int chunk = (int)(bid % jb.chunks);
  const int slab = (int)((bid / jb.chunks) % jb.slabs);
  const int64_t m = bid / ((int64_t)jb.chunks * jb.slabs);

  int vc, r0, rstep;
  if (V >= kThreads) {
    vc = slab * kThreads + threadIdx.x;
    r0 = 0;
    rstep = 1;
  } else {
    rstep = kThreads / V;
    r0 = threadIdx.x / V;
    vc = threadIdx.x - r0 * V;
    if (r0 >= rstep) return;           // lanes beyond the last whole row of a pass idle
  }
  if (vc >= V) return;

  const float *grow = o.g + m * o.ldg + 4 * vc;
  f32x4 gv;
  if (((reinterpret_cast<uintptr_t>(o.g) & 15) == 0) && ((o.ldg & 3) == 0)) {
    gv = *reinterpret_cast<const f32x4 *>(grow);
  } else {
    gv[0] = grow[0]; gv[1] = grow[1]; gv[2] = grow[2]; gv[3] = grow[3];
  }

  const int64_t abase = (m / o.S) * o.lda;
  const int i_begin = chunk * jb.per_chunk;
  const int i_end = min(i_begin + jb.per_chunk, o.d_in);
  f32x4 *obase = reinterpret_cast<f32x4 *>(o.out + m * (int64_t)o.d_in * o.d_out) + vc;

  for (int i = i_begin + r0; i < i_end; i += rstep) {
    const float av = load_a(o.a, o.a_bf16, abase + i);
    __builtin_nontemporal_store(gv * av, obase + (int64_t)i * V);
  }
}

// Any d_out, any alignment: one thread per output value of a flattened [d_in * d_out] iteration.
__device__ __forceinline__ void outer_flat(const OuterJob &jb, int64_t bid) {
  const OuterArgs &o = jb.o;
  const int chunk = (int)(bid % jb.chunks);
  const int64_t m = bid / jb.chunks;
  const int64_t per_m = (int64_t)o.d_in * o.d_out;
  const int64_t e_begin = (int64_t)chunk * jb.per_chunk;
  const int64_t e_end = min(e_begin + jb.per_chunk, per_m);
  const int64_t abase = (m / o.S) * o.lda;
  const float *grow = o.g + m * o.ldg;
  float *obase = o.out + m * per_m;
  for (int64_t e = e_begin + threadIdx.x; e < e_end; e += kThreads) {
    const int i = (int)(e / o.d_out);
    const int j = (int)(e - (int64_t)i * o.d_out);
    obase[e] = load_a(o.a, o.a_bf16, abase + i) * grow[j];
  }
}

// All outer products of one call (one per layer) in a single launch: the workgroup id selects
// the job, so that the short ramp-up and tail of a streaming kernel are paid once per call and
// small layers fill the tail of large ones.
__global__ __launch_bounds__(kThreads) void outer_product_kernel(const OuterBatch batch) {
  const int64_t bid = blockIdx.x;
  int j = 0;
#pragma unroll
  for (int t = 1; t < kMaxJobs; ++t)
    if (t < batch.n && bid >= batch.job[t].block_begin) j = t;
  const OuterJob &jb = batch.job[j];
  if (jb.vec)
    outer_vec4(jb, bid - jb.block_begin);
  else
    outer_flat(jb, bid - jb.block_begin);
}

// Cuts one outer product into workgroups; returns the number of workgroups.
int64_t plan_job(const OuterArgs &o, OuterJob &jb) {
  jb.o = o;
  jb.vec = (o.d_out % 4 == 0) && ((reinterpret_cast<uintptr_t>(o.out) & 15) == 0);
  if (jb.vec) {
    const int V = o.d_out / 4;
    jb.V = V;
    jb.slabs = V >= kThreads ? (V + kThreads - 1) / kThreads : 1;
    const int rows_per_pass = V >= kThreads ? 1 : kThreads / V;
    // about 64 KiB of output per workgroup
    const int64_t pass_bytes = (int64_t)rows_per_pass * (V >= kThreads ? kThreads : V) * 16;
    int passes = (int)((65536 + pass_bytes - 1) / pass_bytes);
    if (passes < 1) passes = 1;
    int rows_per_chunk = passes * rows_per_pass;
    if (rows_per_chunk > o.d_in)
      rows_per_chunk = ((o.d_in + rows_per_pass - 1) / rows_per_pass) * rows_per_pass;
    jb.per_chunk = rows_per_chunk;
    jb.chunks = (o.d_in + rows_per_chunk - 1) / rows_per_chunk;
    return o.M * jb.slabs * jb.chunks;
  }
  const int64_t per_m = (int64_t)o.d_in * o.d_out;
  jb.V = 0;
  jb.slabs = 1;
  jb.per_chunk = 16384;
  jb.chunks = (int)((per_m + jb.per_chunk - 1) / jb.per_chunk);
  return o.M * jb.chunks;
}

}  // namespace

hipError_t launch_outer(const OuterArgs *jobs, int n, hipStream_t stream) {
  int at = 0;
  while (at < n) {
    OuterBatch batch{};
    int64_t blocks = 0;
    while (at < n && batch.n < kMaxJobs) {
      const OuterArgs &o = jobs[at++];
      if (o.M <= 0 || o.d_in <= 0 || o.d_out <= 0) continue;
      OuterJob &jb = batch.job[batch.n];
      const int64_t nb = plan_job(o, jb);
      if (blocks + nb > 0x7fffffffLL) {
        if (batch.n == 0) return hipErrorInvalidConfiguration;   // one job alone is too large
        --at;                                                    // start a new launch with it
        break;
      }
      jb.block_begin = blocks;
      blocks += nb;
      ++batch.n;
    }
    if (batch.n == 0) continue;
    hipLaunchKernelGGL(outer_product_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream,
                       batch);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace pfg
