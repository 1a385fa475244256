// C ABI of the conditional inside a parallel-for: argument checks, workspace layout and the order in
// which the kernels are enqueued.  No arithmetic of the method happens on the host, and no count
// comes back from the device: the products of a branch are launched for all n rows and take the
// number of rows that are really theirs from device memory.
#include <algorithm>

#include "../../include/pfg.h"
#include "common.h"
#include "host.h"

namespace {

using namespace pfg;

constexpr int64_t kMaxCondRows = (int64_t)1 << 24;

struct CondPlan {
  size_t total = 0;
  size_t T = 0, buf0 = 0, buf1 = 0, flags = 0, cnt = 0, rows = 0, meta = 0;
  size_t take(size_t bytes) {
    const size_t at = total;
    total += (bytes + 255) / 256 * 256;
    return at;
  }
};

int hidden_max(const pfg_mlp *m) {
  int w = 1;
  for (int l = 1; l < m->num_layers; ++l) w = std::max(w, m->dims[l]);
  return w;
}

int check_cond(const pfg_cond *net) {
  if (!net) return fail(PFG_ERR_NULL, "net is NULL");
  const pfg_mlp *parts[3] = {&net->pre, &net->then_net, &net->else_net};
  const char *names[3] = {"pre", "then_net", "else_net"};
  for (int i = 0; i < 3; ++i) {
    int rc = check_mlp(parts[i]);
    if (rc) return rc;
    if (parts[i]->dtype != PFG_F32)
      return fail(PFG_ERR_UNSUPPORTED, "%s: the conditional path is float32 only (dtype %d given)", names[i],
                  parts[i]->dtype);
  }
  const int dT = net->pre.dims[net->pre.num_layers];
  if (net->then_net.dims[0] != dT || net->else_net.dims[0] != dT)
    return fail(PFG_ERR_SHAPE, "the branches must take the %d outputs of pre (then_net takes %d, else_net %d)",
                dT, net->then_net.dims[0], net->else_net.dims[0]);
  const int dthen = net->then_net.dims[net->then_net.num_layers];
  const int delse = net->else_net.dims[net->else_net.num_layers];
  if (dthen != delse)
    return fail(PFG_ERR_SHAPE, "the branches must have the same output width (then_net %d, else_net %d)", dthen,
                delse);
  return PFG_OK;
}

int check_cond_rows(const pfg_cond *net, int64_t n) {
  if (n < 1) return fail(PFG_ERR_SHAPE, "n = %lld must be at least 1", (long long)n);
  if (n > kMaxCondRows)
    return fail(PFG_ERR_OVERFLOW, "n = %lld exceeds %lld rows", (long long)n, (long long)kMaxCondRows);
  const pfg_mlp *parts[3] = {&net->pre, &net->then_net, &net->else_net};
  for (const pfg_mlp *m : parts)
    for (int l = 0; l <= m->num_layers; ++l) {
      if (l > 0 && (int64_t)m->dims[l - 1] * m->dims[l] > 0x7fffffffLL)
        return fail(PFG_ERR_OVERFLOW, "a weight matrix of %d x %d exceeds 2^31 - 1 entries", m->dims[l - 1],
                    m->dims[l]);
      if ((int64_t)m->dims[l] > kMaxElems / n)
        return fail(PFG_ERR_OVERFLOW, "%lld rows of width %d exceed the indexing limit", (long long)n,
                    m->dims[l]);
    }
  return PFG_OK;
}

CondPlan make_cond_plan(const pfg_cond *net, int64_t n) {
  const size_t f = sizeof(float);
  const size_t dT = net->pre.dims[net->pre.num_layers];
  const size_t hmax = std::max({hidden_max(&net->pre), hidden_max(&net->then_net), hidden_max(&net->else_net)});
  CondPlan p;
  p.T = p.take(f * n * dT);
  p.buf0 = p.take(f * n * hmax);        // hidden activations, two buffers used alternately
  p.buf1 = p.take(f * n * hmax);
  p.flags = p.take(sizeof(int32_t) * n);
  p.cnt = p.take(sizeof(int32_t) * cond_count_groups(n));
  p.rows = p.take(sizeof(int32_t) * n);
  p.meta = p.take(sizeof(int32_t) * 4);
  return p;
}

int32_t *ws_int(void *ws, size_t off) {
  return reinterpret_cast<int32_t *>(static_cast<char *>(ws) + off);
}

// out = m(in) on n rows (or on the rows of an index set: `sub` = {count, offset} in device memory,
// `rows` the set; the first layer reads its rows of `in` through the set, the last layer stores its
// rows of `out` through it, what lies between is kept densely packed).
int run_mlp(const pfg_mlp *m, const float *in, int64_t n, bool last_act, float *out, float *buf0,
            float *buf1, const int32_t *sub, const int32_t *rows, const char *family, hipStream_t stream) {
  const int L = m->num_layers;
  const int32_t *d = m->dims;
  float *bufs[2] = {buf0, buf1};
  for (int l = 1; l <= L; ++l) {
    GemmArgs g{};
    g.A = (l == 1) ? in : bufs[l & 1];
    g.lda = d[l - 1];
    g.a_batch_stride = d[l - 1];
    g.S = 1;
    g.a_is_f32 = 1;
    g.W = m->W[l - 1];
    g.ldw = d[l];
    g.w_kn = 1;
    g.M = (int32_t)n;
    g.N = d[l];
    g.K = d[l - 1];
    g.bias = (m->b && m->b[l - 1]) ? m->b[l - 1] : nullptr;
    g.act = m->hidden_act;
    g.epilogue = (l < L || last_act) ? EPI_FORWARD : EPI_BIAS;
    g.C = (l == L) ? out : bufs[(l + 1) & 1];
    g.ldc = d[l];
    if (sub) {
      g.sub = sub;
      g.sub_rows = rows;
      g.sub_gather = (l == 1);
      g.sub_scatter = (l == L);
    }
    PFG_LAUNCH(family, launch_gemm(g, stream));
  }
  return PFG_OK;
}

}  // namespace

extern "C" {

int pfg_cond_workspace_bytes(const pfg_cond *net, int64_t n, size_t *bytes) {
  clear_error();
  if (!bytes) return fail(PFG_ERR_NULL, "bytes is NULL");
  int rc = check_cond(net);
  if (rc) return rc;
  if ((rc = check_cond_rows(net, n))) return rc;
  *bytes = make_cond_plan(net, n).total;
  return PFG_OK;
}

int pfg_cond_forward(const pfg_cond *net, const void *X, int64_t n, int invariant_cond, float *R_out,
                     int32_t *cond_out, int32_t *counts_out, void *workspace, size_t workspace_bytes,
                     void *hip_stream) {
  clear_error();
  int rc = check_cond(net);
  if (rc) return rc;
  if ((rc = check_cond_rows(net, n))) return rc;
  if ((rc = check_mlp_weights(&net->pre))) return rc;
  if ((rc = check_mlp_weights(&net->then_net))) return rc;
  if ((rc = check_mlp_weights(&net->else_net))) return rc;
  if (invariant_cond != PFG_COND_PER_ITERATION && invariant_cond != 0 && invariant_cond != 1)
    return fail(PFG_ERR_UNSUPPORTED, "invariant_cond = %d is none of -1, 0, 1", invariant_cond);
  const bool per_iteration = (invariant_cond == PFG_COND_PER_ITERATION);
  if (per_iteration && !net->cond_w) return fail(PFG_ERR_NULL, "net->cond_w is NULL");
  if (!X) return fail(PFG_ERR_NULL, "X is NULL");
  if (!R_out) return fail(PFG_ERR_NULL, "R_out is NULL");
  const CondPlan p = make_cond_plan(net, n);
  if (!workspace) return fail(PFG_ERR_WORKSPACE, "workspace is NULL (%zu bytes needed)", p.total);
  if (reinterpret_cast<uintptr_t>(workspace) & 255)
    return fail(PFG_ERR_WORKSPACE, "workspace is not 256-byte aligned");
  if (workspace_bytes < p.total)
    return fail(PFG_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, p.total);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  void *ws = workspace;
  float *T = ws_at(ws, p.T), *buf0 = ws_at(ws, p.buf0), *buf1 = ws_at(ws, p.buf1);
  const int dT = net->pre.dims[net->pre.num_layers];

  // the part in front of the `if`, for all iterations at once
  if ((rc = run_mlp(&net->pre, static_cast<const float *>(X), n, true, T, buf0, buf1, nullptr, nullptr,
                    "cond_gemm_pre", stream)))
    return rc;

  if (!per_iteration) {
    // loop-invariant condition: one branch, every row, no index sets
    PFG_LAUNCH("cond_partition", launch_cond_invariant((int32_t)n, invariant_cond, cond_out, counts_out, stream));
    return run_mlp(invariant_cond ? &net->then_net : &net->else_net, T, n, false, R_out, buf0, buf1, nullptr,
                   nullptr, invariant_cond ? "cond_gemm_then" : "cond_gemm_else", stream);
  }

  int32_t *meta = ws_int(ws, p.meta), *rows = ws_int(ws, p.rows);
  PFG_LAUNCH("cond_partition",
             launch_cond_partition(T, dT, (int32_t)n, dT, static_cast<const float *>(net->cond_w), net->cond_c,
                                   ws_int(ws, p.flags), ws_int(ws, p.cnt), rows, meta, cond_out, counts_out,
                                   stream));
  if ((rc = run_mlp(&net->then_net, T, n, false, R_out, buf0, buf1, meta, rows, "cond_gemm_then", stream)))
    return rc;
  return run_mlp(&net->else_net, T, n, false, R_out, buf0, buf1, meta + 2, rows, "cond_gemm_else", stream);
}

}  // extern "C"
