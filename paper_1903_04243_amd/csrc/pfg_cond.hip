// C ABI of the conditional inside a parallel-for: argument checks, workspace layout and the order in
// which the kernels are enqueued.  No arithmetic of the method happens on the host, and no count
// comes back from the device: the products of a branch are launched for all n rows and take the
// number of rows that are really theirs from device memory.
#include <algorithm>
#include <vector>

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

// ------------------------------------------------------------------------------------------
// Per-example gradients through the conditional.
// ------------------------------------------------------------------------------------------
struct BranchPlan {
  std::vector<size_t> act, dphi, G;    // hidden layers k = 1 .. L - 1 (entry 0 unused): packed rows of the set
};

struct CondGradPlan {
  size_t total = 0;
  std::vector<size_t> act, dphi, G;    // pre: layers 1 .. L_pre (its last layer is activated too)
  BranchPlan br[2];                    // then, else
  size_t R = 0, dR = 0, GT = 0, flags = 0, cnt = 0, rows = 0, meta = 0;
  size_t take(size_t bytes) {
    const size_t at = total;
    total += (bytes + 255) / 256 * 256;
    return at;
  }
};

CondGradPlan make_cond_grad_plan(const pfg_cond *net, int64_t n) {
  const size_t f = sizeof(float);
  CondGradPlan p;
  const pfg_mlp *pre = &net->pre;
  const int Lp = pre->num_layers;
  p.act.assign(Lp + 1, 0);
  p.dphi.assign(Lp + 1, 0);
  p.G.assign(Lp + 1, 0);
  for (int l = 1; l <= Lp; ++l) {
    p.act[l] = p.take(f * n * pre->dims[l]);
    p.dphi[l] = p.take(f * n * pre->dims[l]);
    p.G[l] = p.take(f * n * pre->dims[l]);
  }
  const pfg_mlp *branch[2] = {&net->then_net, &net->else_net};
  for (int q = 0; q < 2; ++q) {
    const int L = branch[q]->num_layers;
    p.br[q].act.assign(L + 1, 0);
    p.br[q].dphi.assign(L + 1, 0);
    p.br[q].G.assign(L + 1, 0);
    for (int k = 1; k < L; ++k) {
      p.br[q].act[k] = p.take(f * n * branch[q]->dims[k]);
      p.br[q].dphi[k] = p.take(f * n * branch[q]->dims[k]);
      p.br[q].G[k] = p.take(f * n * branch[q]->dims[k]);
    }
  }
  const size_t dout = net->then_net.dims[net->then_net.num_layers];
  p.R = p.take(f * n * dout);
  p.dR = p.take(f * n * dout);
  p.GT = p.take(f * n * pre->dims[Lp]);
  p.flags = p.take(sizeof(int32_t) * n);
  p.cnt = p.take(sizeof(int32_t) * cond_count_groups(n));
  p.rows = p.take(sizeof(int32_t) * n);
  p.meta = p.take(sizeof(int32_t) * 4);
  return p;
}

GemmArgs dense_gemm(const float *A, int64_t lda, const void *W, int64_t ldw, int w_kn, int64_t M, int N, int K) {
  GemmArgs g{};
  g.A = A; g.lda = lda; g.a_batch_stride = lda; g.S = 1; g.a_is_f32 = 1;
  g.W = W; g.ldw = ldw; g.w_kn = w_kn;
  g.M = (int32_t)M; g.N = N; g.K = K;
  return g;
}

}  // namespace

extern "C" {

int pfg_cond_grads_workspace_bytes(const pfg_cond *net, int64_t n, size_t *bytes) {
  clear_error();
  if (!bytes) return fail(PFG_ERR_NULL, "bytes is NULL");
  int rc = check_cond(net);
  if (rc) return rc;
  if ((rc = check_cond_rows(net, n))) return rc;
  *bytes = make_cond_grad_plan(net, n).total;
  return PFG_OK;
}

int pfg_cond_per_example_grads(const pfg_cond *net, const void *X, const int32_t *labels, int64_t n,
                               int invariant_cond, float *const *dW_pre_out, float *const *db_pre_out,
                               float *const *dW_then_out, float *const *db_then_out,
                               float *const *dW_else_out, float *const *db_else_out, float *loss_out,
                               int32_t *cond_out, int32_t *counts_out, void *workspace,
                               size_t workspace_bytes, void *hip_stream) {
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
  if (!labels) return fail(PFG_ERR_NULL, "labels is NULL");
  const pfg_mlp *pre = &net->pre;
  const pfg_mlp *branch[2] = {&net->then_net, &net->else_net};
  float *const *dW_br[2] = {dW_then_out, dW_else_out};
  float *const *db_br[2] = {db_then_out, db_else_out};
  // every stacked gradient must stay within the index range of the writer
  const pfg_mlp *parts[3] = {pre, branch[0], branch[1]};
  for (const pfg_mlp *m : parts)
    for (int l = 1; l <= m->num_layers; ++l)
      if ((int64_t)m->dims[l - 1] * m->dims[l] > kMaxElems / n)
        return fail(PFG_ERR_OVERFLOW, "%lld x %d x %d gradient values exceed the indexing limit", (long long)n,
                    m->dims[l - 1], m->dims[l]);
  const CondGradPlan p = make_cond_grad_plan(net, n);
  if (!workspace) return fail(PFG_ERR_WORKSPACE, "workspace is NULL (%zu bytes needed)", p.total);
  if (reinterpret_cast<uintptr_t>(workspace) & 255)
    return fail(PFG_ERR_WORKSPACE, "workspace is not 256-byte aligned");
  if (workspace_bytes < p.total)
    return fail(PFG_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, p.total);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  void *ws = workspace;
  const int Lp = pre->num_layers;
  const int dT = pre->dims[Lp], dout = branch[0]->dims[branch[0]->num_layers];
  auto bias_of = [](const pfg_mlp *m, int l) -> const void * { return (m->b && m->b[l - 1]) ? m->b[l - 1] : nullptr; };

  // ---- the part in front of the `if`, all rows, every layer kept (its last layer is activated too) ----
  for (int l = 1; l <= Lp; ++l) {
    GemmArgs g = dense_gemm(l == 1 ? static_cast<const float *>(X) : ws_at(ws, p.act[l - 1]), pre->dims[l - 1],
                            pre->W[l - 1], pre->dims[l], 1, n, pre->dims[l], pre->dims[l - 1]);
    g.bias = bias_of(pre, l); g.act = pre->hidden_act; g.epilogue = EPI_FORWARD;
    g.C = ws_at(ws, p.act[l]); g.C2 = ws_at(ws, p.dphi[l]); g.ldc = pre->dims[l];
    PFG_LAUNCH("cond_gemm_pre", launch_gemm(g, stream));
  }
  const float *T = ws_at(ws, p.act[Lp]);

  // ---- the index sets (for a loop-invariant condition: one set holds every row) ----
  int32_t *meta = ws_int(ws, p.meta), *rows = ws_int(ws, p.rows);
  if (per_iteration) {
    PFG_LAUNCH("cond_partition",
               launch_cond_partition(T, dT, (int32_t)n, dT, static_cast<const float *>(net->cond_w), net->cond_c,
                                     ws_int(ws, p.flags), ws_int(ws, p.cnt), rows, meta, cond_out, counts_out,
                                     stream));
  } else {
    PFG_LAUNCH("cond_partition", launch_cond_identity_list(rows, meta, (int32_t)n, invariant_cond, stream));
    PFG_LAUNCH("cond_partition", launch_cond_invariant((int32_t)n, invariant_cond, cond_out, counts_out, stream));
  }

  // ---- each branch forward on the rows of its set: hidden layers packed, results put back at
  // their rows of R ----
  float *R = ws_at(ws, p.R), *dR = ws_at(ws, p.dR);
  for (int q = 0; q < 2; ++q) {
    const pfg_mlp *m = branch[q];
    const int L = m->num_layers;
    const char *family = q == 0 ? "cond_gemm_then" : "cond_gemm_else";
    for (int k = 1; k <= L; ++k) {
      GemmArgs g = dense_gemm(k == 1 ? T : ws_at(ws, p.br[q].act[k - 1]), m->dims[k - 1], m->W[k - 1], m->dims[k], 1,
                              n, m->dims[k], m->dims[k - 1]);
      g.bias = bias_of(m, k); g.act = m->hidden_act; g.ldc = m->dims[k];
      g.sub = meta + 2 * q; g.sub_rows = rows; g.sub_gather = (k == 1); g.sub_scatter = (k == L);
      if (k < L) {
        g.epilogue = EPI_FORWARD; g.C = ws_at(ws, p.br[q].act[k]); g.C2 = ws_at(ws, p.br[q].dphi[k]);
      } else {
        g.epilogue = EPI_BIAS; g.C = R;
      }
      PFG_LAUNCH(family, launch_gemm(g, stream));
    }
  }

  // ---- every iteration's own loss and its cotangent at r ----
  PFG_LAUNCH("head", launch_head_softmax_ce(R, labels, n, dout, dR, loss_out, stream));

  // ---- each branch in reverse on its rows; the cotangent of t goes back to the rows of G_T ----
  float *GT = ws_at(ws, p.GT);
  for (int q = 0; q < 2; ++q) {
    const pfg_mlp *m = branch[q];
    const int L = m->num_layers;
    const char *family = q == 0 ? "cond_gemm_then_reverse" : "cond_gemm_else_reverse";
    for (int k = L; k >= 1; --k) {
      // A = G_k: the rows of dR gathered through the set for the top layer, packed below it
      GemmArgs g = dense_gemm(k == L ? dR : ws_at(ws, p.br[q].G[k]), m->dims[k], m->W[k - 1], m->dims[k], 0, n,
                              m->dims[k - 1], m->dims[k]);
      g.sub = meta + 2 * q; g.sub_rows = rows; g.sub_gather = (k == L);
      if (k > 1) {
        g.epilogue = EPI_MASK; g.emask = ws_at(ws, p.br[q].dphi[k - 1]); g.ld_emask = m->dims[k - 1];
        g.C = ws_at(ws, p.br[q].G[k - 1]); g.ldc = m->dims[k - 1];
      } else {
        g.epilogue = EPI_NONE; g.C = GT; g.ldc = dT; g.sub_scatter = 1;
      }
      PFG_LAUNCH(family, launch_gemm(g, stream));
    }
  }

  // ---- the shared part in reverse, all rows: G_Lp = G_T * phi'(z_Lp), then the usual chain ----
  std::vector<float *> G(Lp + 1, nullptr);
  for (int l = 1; l <= Lp; ++l) G[l] = (db_pre_out && db_pre_out[l - 1]) ? db_pre_out[l - 1] : ws_at(ws, p.G[l]);
  PFG_LAUNCH("cond_mask", launch_scale_rows(GT, 0, dT, dT, ws_at(ws, p.dphi[Lp]), dT, n, 1, dT, G[Lp], dT, stream));
  for (int l = Lp; l >= 2; --l) {
    GemmArgs g = dense_gemm(G[l], pre->dims[l], pre->W[l - 1], pre->dims[l], 0, n, pre->dims[l - 1], pre->dims[l]);
    g.epilogue = EPI_MASK; g.emask = ws_at(ws, p.dphi[l - 1]); g.ld_emask = pre->dims[l - 1];
    g.C = G[l - 1]; g.ldc = pre->dims[l - 1];
    PFG_LAUNCH("cond_gemm_pre_reverse", launch_gemm(g, stream));
  }

  // ---- bias gradients of the branches: the cotangent rows put back at their iterations, zeros for
  // the iterations of the other set ----
  for (int q = 0; q < 2; ++q) {
    const pfg_mlp *m = branch[q];
    const int L = m->num_layers;
    for (int k = 1; k <= L; ++k) {
      if (!db_br[q] || !db_br[q][k - 1]) continue;
      PFG_LAUNCH("cond_scatter",
                 launch_cond_scatter_rows(k == L ? dR : ws_at(ws, p.br[q].G[k]), m->dims[k], k == L, rows,
                                          meta + 2 * q, (int32_t)n, m->dims[k], db_br[q][k - 1], m->dims[k], stream));
    }
  }

  // ---- the outer products: the shared part's layers in one launch over all rows, the branches'
  // layers in one launch over the list (an iteration outside a branch's set gets zeros) ----
  std::vector<OuterArgs> jobs;
  for (int l = 1; l <= Lp; ++l) {
    if (!dW_pre_out || !dW_pre_out[l - 1]) continue;
    OuterArgs o{};
    o.a = l == 1 ? X : ws_at(ws, p.act[l - 1]); o.lda = pre->dims[l - 1];
    o.g = G[l]; o.ldg = pre->dims[l];
    o.out = dW_pre_out[l - 1]; o.M = n; o.S = 1; o.d_in = pre->dims[l - 1]; o.d_out = pre->dims[l];
    jobs.push_back(o);
  }
  for (int q = 0; q < 2; ++q) {
    const pfg_mlp *m = branch[q];
    const int L = m->num_layers;
    for (int k = 1; k <= L; ++k) {
      if (!dW_br[q] || !dW_br[q][k - 1]) continue;
      OuterArgs o{};
      o.a = k == 1 ? T : ws_at(ws, p.br[q].act[k - 1]); o.lda = m->dims[k - 1]; o.a_gather = (k == 1);
      o.g = k == L ? dR : ws_at(ws, p.br[q].G[k]); o.ldg = m->dims[k]; o.g_gather = (k == L);
      o.out = dW_br[q][k - 1]; o.M = n; o.S = 1; o.d_in = m->dims[k - 1]; o.d_out = m->dims[k];
      o.sub = meta + 2 * q; o.sub_rows = rows;
      jobs.push_back(o);
    }
  }
  if (!jobs.empty()) PFG_LAUNCH("outer_product", launch_outer(jobs.data(), (int)jobs.size(), stream));
  return PFG_OK;
}

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
