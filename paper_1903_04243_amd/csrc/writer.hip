// Per-instance outer-product writer:  out[m, i, j] = a[m / S, i] * g[m, j].
//
// Section 3.4: a matmul whose operands are BOTH loop-variant becomes a batch_matmul over the
// stacked iterations.  The weight gradient of one iteration is the [d_in, 1] x [1, d_out] product
// of the layer input and the cotangent row, a contraction of length one, so the "batched matmul"
// degenerates into one multiply per output value and the kernel is bound by how fast HBM absorbs
// the stacked [M, d_in, d_out] result.  It is therefore a pure streaming writer: every lane holds
// four consecutive g values in registers, multiplies them by one a value per row and issues one
// 16-byte non-temporal store per row; consecutive lanes cover consecutive 16-byte pieces of a row
// and a workgroup walks a contiguous run of rows of one iteration m.
#include "common.h"

namespace pfg {

namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ float load_a(const void *a, int a_bf16, int64_t idx) {
  if (a_bf16) return (float)static_cast<const __bf16 *>(a)[idx];
  return static_cast<const float *>(a)[idx];
}

// d_out % 4 == 0, out 16-byte aligned.  V = d_out / 4 vector columns.
// Workgroup = (m, column slab of up to 256 vectors, chunk of rows).  When V < 256 a pass covers
// 256 / V rows at once.
__global__ __launch_bounds__(kThreads) void outer_vec4_kernel(const OuterArgs o, int V,
                                                              int slabs, int row_chunks,
                                                              int rows_per_chunk) {
  const int64_t bid = blockIdx.x;
  const int chunk = (int)(bid % row_chunks);
  const int slab = (int)((bid / row_chunks) % slabs);
  const int64_t m = bid / ((int64_t)row_chunks * slabs);

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
  const int i_begin = chunk * rows_per_chunk;
  const int i_end = min(i_begin + rows_per_chunk, o.d_in);
  f32x4 *obase = reinterpret_cast<f32x4 *>(o.out + m * (int64_t)o.d_in * o.d_out) + vc;

  for (int i = i_begin + r0; i < i_end; i += rstep) {
    const float av = load_a(o.a, o.a_bf16, abase + i);
    __builtin_nontemporal_store(gv * av, obase + (int64_t)i * V);
  }
}

// Any d_out, any alignment: one thread per output value of a flattened [d_in * d_out] iteration.
__global__ __launch_bounds__(kThreads) void outer_flat_kernel(const OuterArgs o, int chunks,
                                                              int per_chunk) {
  const int64_t bid = blockIdx.x;
  const int chunk = (int)(bid % chunks);
  const int64_t m = bid / chunks;
  const int64_t per_m = (int64_t)o.d_in * o.d_out;
  const int64_t e_begin = (int64_t)chunk * per_chunk;
  const int64_t e_end = min(e_begin + per_chunk, per_m);
  const int64_t abase = (m / o.S) * o.lda;
  const float *grow = o.g + m * o.ldg;
  float *obase = o.out + m * per_m;
  for (int64_t e = e_begin + threadIdx.x; e < e_end; e += kThreads) {
    const int i = (int)(e / o.d_out);
    const int j = (int)(e - (int64_t)i * o.d_out);
    obase[e] = load_a(o.a, o.a_bf16, abase + i) * grow[j];
  }
}

}  // namespace

hipError_t launch_outer(const OuterArgs &o, hipStream_t stream) {
  if (o.M <= 0 || o.d_in <= 0 || o.d_out <= 0) return hipSuccess;
  const bool vec = (o.d_out % 4 == 0) && ((reinterpret_cast<uintptr_t>(o.out) & 15) == 0);
  if (vec) {
    const int V = o.d_out / 4;
    const int slabs = V >= kThreads ? (V + kThreads - 1) / kThreads : 1;
    const int rows_per_pass = V >= kThreads ? 1 : kThreads / V;
    // about 64 KiB of output per workgroup
    const int64_t pass_bytes = (int64_t)rows_per_pass * (V >= kThreads ? kThreads : V) * 16;
    int passes = (int)((65536 + pass_bytes - 1) / pass_bytes);
    if (passes < 1) passes = 1;
    int rows_per_chunk = passes * rows_per_pass;
    if (rows_per_chunk > o.d_in) rows_per_chunk = ((o.d_in + rows_per_pass - 1) / rows_per_pass) * rows_per_pass;
    const int row_chunks = (o.d_in + rows_per_chunk - 1) / rows_per_chunk;
    const int64_t blocks = o.M * slabs * row_chunks;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(outer_vec4_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, o, V,
                       slabs, row_chunks, rows_per_chunk);
  } else {
    const int64_t per_m = (int64_t)o.d_in * o.d_out;
    const int per_chunk = 16384;
    const int chunks = (int)((per_m + per_chunk - 1) / per_chunk);
    const int64_t blocks = o.M * chunks;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(outer_flat_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, o,
                       chunks, per_chunk);
  }
  return hipGetLastError();
}

}  // namespace pfg
