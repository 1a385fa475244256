// C ABI of libpfg: argument checks, workspace layout and the order in which the kernels of the
// three operations are enqueued.  No arithmetic of the method happens on the host.
#include <algorithm>
#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/pfg.h"
#include "common.h"
#include "host.h"

namespace {
thread_local char g_err[512] = "";
thread_local const char *t_family = "kernel";   // family name of the launches being enqueued
}  // namespace

namespace pfg {
int fail(int code, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}
void clear_error() { g_err[0] = 0; }
void set_timing_family(const char *name) { t_family = name; }
}  // namespace pfg

namespace {

using namespace pfg;

// ------------------------------------------------------------------------------------------
// Per-kernel timing: every kernel launch gets its own pair of events attached to the dispatch
// (see PFG_KERNEL); their difference is the kernel's run time on the device.
// ------------------------------------------------------------------------------------------
struct TimedLaunch { const char *name; hipEvent_t start, stop; };
std::mutex g_timing_mu;
std::atomic<bool> g_timing_on{false};
std::vector<TimedLaunch> g_pending;
std::map<std::string, std::pair<int64_t, double>> g_totals;
void drain_pending() {
  std::lock_guard<std::mutex> lk(g_timing_mu);
  for (auto &t : g_pending) {
    float ms = 0.f;
    if (hipEventSynchronize(t.stop) == hipSuccess &&
        hipEventElapsedTime(&ms, t.start, t.stop) == hipSuccess) {
      auto &e = g_totals[t.name];
      e.first += 1;
      e.second += ms;
    }
    (void)hipEventDestroy(t.start);
    (void)hipEventDestroy(t.stop);
  }
  g_pending.clear();
}

}  // namespace

namespace pfg {
bool timing_next_events(hipEvent_t *start, hipEvent_t *stop) {
  if (!g_timing_on.load(std::memory_order_relaxed)) return false;
  if (hipEventCreate(start) != hipSuccess) return false;
  if (hipEventCreate(stop) != hipSuccess) { (void)hipEventDestroy(*start); return false; }
  std::lock_guard<std::mutex> lk(g_timing_mu);
  g_pending.push_back({t_family, *start, *stop});
  return true;
}
}  // namespace pfg

namespace {

// ------------------------------------------------------------------------------------------
// Validation helpers.
// ------------------------------------------------------------------------------------------
constexpr int kMaxLayers = 256;
constexpr int64_t kMaxDim = 1 << 24;

int check_net(const pfg_mlp *net) {
  if (!net) return fail(PFG_ERR_NULL, "net is NULL");
  if (net->num_layers < 1 || net->num_layers > kMaxLayers)
    return fail(PFG_ERR_SHAPE, "num_layers = %d is outside [1, %d]", net->num_layers, kMaxLayers);
  if (!net->dims) return fail(PFG_ERR_NULL, "net->dims is NULL");
  for (int l = 0; l <= net->num_layers; ++l)
    if (net->dims[l] < 1 || net->dims[l] > kMaxDim)
      return fail(PFG_ERR_SHAPE, "dims[%d] = %d is outside [1, %lld]", l, net->dims[l],
                  (long long)kMaxDim);
  if (net->hidden_act < PFG_ACT_IDENTITY || net->hidden_act > PFG_ACT_GELU_ERF)
    return fail(PFG_ERR_UNSUPPORTED, "unknown activation %d", net->hidden_act);
  if (net->dtype != PFG_F32 && net->dtype != PFG_BF16)
    return fail(PFG_ERR_UNSUPPORTED, "unknown dtype %d", net->dtype);
  return PFG_OK;
}

int check_weights(const pfg_mlp *net) {
  if (!net->W) return fail(PFG_ERR_NULL, "net->W is NULL");
  for (int l = 0; l < net->num_layers; ++l)
    if (!net->W[l]) return fail(PFG_ERR_NULL, "net->W[%d] is NULL", l);
  return PFG_OK;
}

}  // namespace

namespace pfg {
int check_mlp(const pfg_mlp *net) { return check_net(net); }
int check_mlp_weights(const pfg_mlp *net) { return check_weights(net); }
}  // namespace pfg

namespace {

int check_rows(int64_t B, int64_t S) {
  if (B < 1) return fail(PFG_ERR_SHAPE, "B = %lld must be at least 1", (long long)B);
  if (S < 1) return fail(PFG_ERR_SHAPE, "S = %lld must be at least 1", (long long)S);
  if (B > kMaxRows || S > kMaxRows || B * S > kMaxRows)
    return fail(PFG_ERR_OVERFLOW, "B * S = %lld * %lld exceeds %lld rows", (long long)B,
                (long long)S, (long long)kMaxRows);
  return PFG_OK;
}

int check_elems(const pfg_mlp *net, int64_t rows) {
  for (int l = 1; l <= net->num_layers; ++l) {
    const int64_t per = (int64_t)net->dims[l - 1] * net->dims[l];
    if (per > 0x7fffffffLL)
      return fail(PFG_ERR_OVERFLOW, "layer %d: %d x %d weights exceed 2^31 - 1 per iteration", l,
                  net->dims[l - 1], net->dims[l]);
    if (per > kMaxElems / rows)
      return fail(PFG_ERR_OVERFLOW, "layer %d: %lld x %d x %d values exceed the indexing limit", l,
                  (long long)rows, net->dims[l - 1], net->dims[l]);
  }
  return PFG_OK;
}

int check_seeds(const pfg_mlp *net, const float *seeds, int64_t S, int64_t stride) {
  const int dL = net->dims[net->num_layers];
  if (!seeds) {
    if (S != dL)
      return fail(PFG_ERR_SHAPE, "identity seeds (seeds == NULL) need S == d_L, got S = %lld, d_L = %d",
                  (long long)S, dL);
    return PFG_OK;
  }
  if (stride != 0 && stride < S * dL)
    return fail(PFG_ERR_SHAPE, "seed_batch_stride = %lld must be 0 or at least S * d_L = %lld",
                (long long)stride, (long long)(S * dL));
  return PFG_OK;
}

int check_hessian(const pfg_mlp *net, int64_t B, int64_t S) {
  const int64_t n = net->dims[0];
  int64_t ktot = 0;
  for (int l = 1; l < net->num_layers; ++l) ktot += net->dims[l];
  if (n * n > 0x7fffffffLL || S * n > kMaxRows || B * n > kMaxRows || ktot > 0x7fffffffLL)
    return fail(PFG_ERR_OVERFLOW, "d_0 = %lld is too wide for B = %lld, S = %lld", (long long)n,
                (long long)B, (long long)S);
  if (n * n > kMaxElems / (B * S) || (ktot && B * (n > S ? n : S) > kMaxElems / ktot))
    return fail(PFG_ERR_OVERFLOW, "B * S * d_0 * d_0 = %lld * %lld * %lld^2 values exceed the indexing limit",
                (long long)B, (long long)S, (long long)n);
  return PFG_OK;
}

// ------------------------------------------------------------------------------------------
// Workspace layout.  Every block is 256-byte aligned.
// ------------------------------------------------------------------------------------------
struct Plan {
  size_t total = 0;
  std::vector<size_t> act, dphi, d2phi, G;   // indexed by layer l (1-based; entry 0 unused)
  size_t logits = 0, P = 0, ping = 0, pong = 0, sq = 0, U = 0, Cc = 0;
  size_t splitk = 0;                  // partial results of a product cut along its contraction, or 0
  size_t head_part = 0;               // partial logits of a head whose contraction is cut, or 0
  int64_t ktot = 0;                   // Hessian: sum of the hidden widths
  std::vector<int64_t> koff;          // Hessian: column offset of hidden layer l in U and Cc
  size_t take(size_t bytes) {
    const size_t at = total;
    total += (bytes + 255) / 256 * 256;
    return at;
  }
};

Plan make_plan(const pfg_mlp *net, int op, int64_t B, int64_t S) {
  const int L = net->num_layers;
  const int32_t *d = net->dims;
  Plan p;
  p.act.assign(L + 1, 0);
  p.dphi.assign(L + 1, 0);
  p.G.assign(L + 1, 0);
  p.d2phi.assign(L + 1, 0);
  p.koff.assign(L + 1, 0);
  const int hidden_last = L - 1;
  for (int l = 1; l <= hidden_last; ++l) {
    p.act[l] = p.take(sizeof(float) * B * d[l]);
    p.dphi[l] = p.take(sizeof(float) * B * d[l]);
  }
  if (op == PFG_OP_HESSIAN_INPUT) {
    size_t widest = 1;
    for (int l = 1; l <= hidden_last; ++l) {
      p.d2phi[l] = p.take(sizeof(float) * B * d[l]);
      p.koff[l] = p.ktot;
      p.ktot += d[l];
      widest = widest > (size_t)d[l] ? widest : (size_t)d[l];
    }
    if (hidden_last >= 1) {
      p.U = p.take(sizeof(float) * B * d[0] * p.ktot);     // tangents [B * d_0, ktot]
      p.Cc = p.take(sizeof(float) * B * S * p.ktot);       // curvature weights [B * S, ktot]
      p.P = p.take(sizeof(float) * S * d[L - 1]);
      p.ping = p.take(sizeof(float) * B * S * widest);
      p.pong = p.take(sizeof(float) * B * S * widest);
    }
  } else if (op == PFG_OP_JACOBIAN_INPUT) {
    size_t widest = 0;
    for (int l = 1; l <= hidden_last; ++l) widest = widest > (size_t)d[l] ? widest : (size_t)d[l];
    // loop-invariant seed block: [S, d_{L-1}] after the first step, or the [S, d_L] identity of
    // a one-layer network
    p.P = p.take(sizeof(float) * S * (L >= 2 ? d[L - 1] : d[L]));
    // two folded cotangent blocks [B * S, widest hidden width] used alternately
    p.ping = p.take(sizeof(float) * B * S * (widest ? widest : 1));
    p.pong = p.take(sizeof(float) * B * S * (widest ? widest : 1));
  } else {
    const int64_t rows = (op == PFG_OP_JACOBIAN_WEIGHTS) ? B * S : B;
    p.logits = p.take(sizeof(float) * B * d[L]);
    for (int l = 1; l <= L; ++l) p.G[l] = p.take(sizeof(float) * rows * d[l]);
    if (op == PFG_OP_GRAD_NORMS) p.sq = p.take(sizeof(float) * B * L);
    if (rows == B && L >= 2) {
      const int z = head_split_shape(B, d[L], d[L - 1]);
      if (z > 1) p.head_part = p.take(sizeof(float) * z * B * d[L]);
    }
    if (rows == B) {
      // the largest [Z, B, width] block a forward layer needs
      size_t most = 0;
      for (int l = 1; l <= L; ++l) {
        const int z = split_k_shape(B, d[l], d[l - 1], net->dtype == PFG_BF16);
        if (z > 1) most = std::max(most, sizeof(float) * z * B * d[l]);
      }
      if (most) p.splitk = p.take(most);
    }
  }
  if (p.total == 0) p.total = 256;
  return p;
}

int check_workspace(const Plan &p, void *ws, size_t bytes) {
  if (!ws) return fail(PFG_ERR_WORKSPACE, "workspace is NULL (%zu bytes needed)", p.total);
  if (reinterpret_cast<uintptr_t>(ws) & 255)
    return fail(PFG_ERR_WORKSPACE, "workspace is not 256-byte aligned");
  if (bytes < p.total)
    return fail(PFG_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", bytes, p.total);
  return PFG_OK;
}

inline float *at(void *ws, size_t off) { return reinterpret_cast<float *>(static_cast<char *>(ws) + off); }

const void *bias_of(const pfg_mlp *net, int l) { return net->b ? net->b[l - 1] : nullptr; }

// Stacked forward pass through layers 1..upto.  Hidden layers store a_l and phi'(z_l); layer L
// (if reached) stores the logits.
struct HeadFusion {      // softmax cross-entropy folded into the last forward layer
  const int32_t *labels;
  float *delta;          // [B, d_L]
  float *loss;           // [B] or nullptr
  float *g_prev;         // [B, d_{L-1}]: also take the cotangent step through layer L, or nullptr
};

int forward(const pfg_mlp *net, const void *X, int64_t B, int upto, void *ws, const Plan &p,
            bool keep_last_hidden_act, hipStream_t stream, const HeadFusion *head = nullptr) {
  const int L = net->num_layers;
  const int32_t *d = net->dims;
  for (int l = 1; l <= upto; ++l) {
    GemmArgs g{};
    g.A = (l == 1) ? X : at(ws, p.act[l - 1]);
    g.lda = d[l - 1];
    g.a_batch_stride = d[l - 1];
    g.S = 1;
    g.a_is_f32 = (l == 1) ? (net->dtype == PFG_F32) : 1;
    g.W = net->W[l - 1];
    g.ldw = d[l];
    g.w_kn = 1;
    g.bf16 = (net->dtype == PFG_BF16);
    g.M = (int32_t)B;
    g.N = d[l];
    g.K = d[l - 1];
    g.bias = bias_of(net, l);
    g.act = net->hidden_act;
    g.ldc = d[l];
    if (l < L) {
      g.epilogue = EPI_FORWARD;
      g.C = (l == upto && !keep_last_hidden_act) ? nullptr : at(ws, p.act[l]);
      g.C2 = at(ws, p.dphi[l]);
    } else if (head) {
      g.epilogue = EPI_HEAD;
      g.C = nullptr;
      g.C2 = head->delta;
      g.labels = head->labels;
      g.loss = head->loss;
      if (head->g_prev && L >= 2) {
        g.head_gprev = head->g_prev;
        g.head_mask = at(ws, p.dphi[L - 1]);
      }
    } else {
      g.epilogue = EPI_BIAS;
      g.C = at(ws, p.logits);
    }
    const int Z = p.splitk ? split_k_factor(g) : 1;
    const int Zh = (p.head_part && g.epilogue == EPI_HEAD) ? head_split_pieces(g) : 1;
    if (g.epilogue == EPI_HEAD && head_rows_applies(g))
      PFG_LAUNCH("gemm_forward", launch_head_rows(g, 0, stream));
    else if (Zh > 1)
      PFG_LAUNCH("gemm_forward", launch_head_split(g, Zh, at(ws, p.head_part), stream));
    else if (Z > 1)
      PFG_LAUNCH("gemm_forward", launch_gemm_split(g, Z, at(ws, p.splitk), stream));
    else
      PFG_LAUNCH("gemm_forward", launch_gemm(g, stream));
  }
  return PFG_OK;
}

// G_{l-1} = (G_l W_l^T) * phi'(z_{l-1}) on the folded rows m = b * S + s.
int cotangent_step(const pfg_mlp *net, int l, const float *G_l, int64_t rows, int64_t S,
                   float *G_prev, void *ws, const Plan &p, hipStream_t stream) {
  const int32_t *d = net->dims;
  GemmArgs g{};
  g.A = G_l;
  g.lda = d[l];
  g.a_batch_stride = S * d[l];
  g.S = (int32_t)S;
  g.a_is_f32 = 1;
  g.W = net->W[l - 1];
  g.ldw = d[l];
  g.w_kn = 0;
  g.bf16 = (net->dtype == PFG_BF16);
  g.M = (int32_t)rows;
  g.N = d[l - 1];
  g.K = d[l];
  g.epilogue = EPI_MASK;
  g.emask = at(ws, p.dphi[l - 1]);
  g.ld_emask = d[l - 1];
  g.C = G_prev;
  g.ldc = d[l - 1];
  PFG_LAUNCH("gemm_cotangent", launch_gemm(g, stream));
  return PFG_OK;
}

OuterArgs outer_job(const pfg_mlp *net, int l, const void *X, const float *G_l, int64_t rows,
                    int64_t S, float *out, void *ws, const Plan &p) {
  const int32_t *d = net->dims;
  OuterArgs o{};
  o.a = (l == 1) ? X : at(ws, p.act[l - 1]);
  o.lda = d[l - 1];
  o.a_bf16 = (l == 1) && (net->dtype == PFG_BF16);
  o.g = G_l;
  o.ldg = d[l];
  o.out = out;
  o.M = rows;
  o.S = (int32_t)S;
  o.d_in = d[l - 1];
  o.d_out = d[l];
  return o;
}

// Backward sweep shared by the two weight-gradient operations: G_L is already in place.  The
// cotangent chain runs first; the outer products of all requested layers then go out together.
int lowest_requested(const pfg_mlp *net, float *const *W_out, float *const *b_out) {
  for (int l = 1; l <= net->num_layers; ++l)
    if ((W_out && W_out[l - 1]) || (b_out && b_out[l - 1])) return l;
  return net->num_layers + 1;
}

int weight_sweep(const pfg_mlp *net, const void *X, int64_t B, int64_t S, float *const *W_out,
                 float *const *b_out, std::vector<float *> &G, void *ws, const Plan &p,
                 hipStream_t stream, bool top_step_done = false) {
  const int L = net->num_layers;
  const int lowest = lowest_requested(net, W_out, b_out);
  for (int l = top_step_done ? L - 1 : L; l > lowest; --l) {
    int rc = cotangent_step(net, l, G[l], B * S, S, G[l - 1], ws, p, stream);
    if (rc) return rc;
  }
  // largest layer first, so that the small ones fill the tail of the launch
  std::vector<OuterArgs> jobs;
  for (int l = 1; l <= L; ++l)
    if (W_out && W_out[l - 1]) jobs.push_back(outer_job(net, l, X, G[l], B * S, S, W_out[l - 1], ws, p));
  std::stable_sort(jobs.begin(), jobs.end(), [](const OuterArgs &x, const OuterArgs &y) {
    return (int64_t)x.d_in * x.d_out > (int64_t)y.d_in * y.d_out;
  });
  if (!jobs.empty())
    PFG_LAUNCH("outer_product", launch_outer(jobs.data(), (int)jobs.size(), stream));
  return PFG_OK;
}

}  // namespace

// Device memory of pfg_per_example_grads_static: what the other entry points take as their
// workspace argument (activations, masks, cotangents, partial products).  One copy per GPU, held
// from the moment the library is loaded on it until the process ends.  The name below is only a
// host-side handle; the address on the current GPU comes from hipGetSymbolAddress.
static __device__ __align__(256) unsigned char scratch[PFG_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};

// Address of `scratch` on the current device, looked up once per device.
int static_scratch(void **out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(PFG_ERR_DEVICE, "hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fail(PFG_ERR_DEVICE, "device index %d is outside [0, %d)", dev, kMaxDevices);
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void *ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr)
      return fail(PFG_ERR_DEVICE, "hipGetSymbolAddress(scratch) on device %d: %s", dev, hipGetErrorString(e));
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return PFG_OK;
}

int per_example_grads_impl(const pfg_mlp *net, const void *X, const int32_t *labels, int64_t B,
                           float *const *dW_out, float *const *db_out, float *loss_out,
                           void *workspace, size_t workspace_bytes, bool use_static,
                           void *hip_stream) {
  g_err[0] = 0;
  int rc = check_net(net);
  if (rc) return rc;
  if ((rc = check_weights(net))) return rc;
  if (!X) return fail(PFG_ERR_NULL, "X is NULL");
  if (!labels) return fail(PFG_ERR_NULL, "labels is NULL");
  if ((rc = check_rows(B, 1))) return rc;
  if ((rc = check_elems(net, B))) return rc;
  const Plan p = make_plan(net, PFG_OP_PER_EXAMPLE_GRADS, B, 1);
  if (use_static) {
    if (p.total > (size_t)PFG_STATIC_SCRATCH_BYTES)
      return fail(PFG_ERR_WORKSPACE,
                  "this network and batch need %zu bytes of scratch memory, the built-in buffer holds %zu: "
                  "use pfg_per_example_grads with a workspace", p.total, (size_t)PFG_STATIC_SCRATCH_BYTES);
    if ((rc = static_scratch(&workspace))) return rc;
    workspace_bytes = PFG_STATIC_SCRATCH_BYTES;
  }
  if ((rc = check_workspace(p, workspace, workspace_bytes))) return rc;

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const int L = net->num_layers;
  const int32_t *d = net->dims;

  // delta_l lives in the caller's db_out[l-1] when given (db_l = delta_l), else in the workspace
  std::vector<float *> G(L + 1, nullptr);
  for (int l = 1; l <= L; ++l)
    G[l] = (db_out && db_out[l - 1]) ? db_out[l - 1] : at(workspace, p.G[l]);

  bool top_step_done = false;
  if (d[L] <= 32) {
    // a whole row of logits fits one output tile: the loss head, and the cotangent step through
    // the last layer if a lower layer's gradient is wanted, ride on the last forward layer
    top_step_done = (L >= 2) && (lowest_requested(net, dW_out, db_out) < L);
    const HeadFusion hf{labels, G[L], loss_out, top_step_done ? G[L - 1] : nullptr};
    if ((rc = forward(net, X, B, L, workspace, p, true, stream, &hf))) return rc;
  } else {
    if ((rc = forward(net, X, B, L, workspace, p, true, stream))) return rc;
    PFG_LAUNCH("head", launch_head_softmax_ce(at(workspace, p.logits), labels, B, d[L], G[L],
                                              loss_out, stream));
  }
  return weight_sweep(net, X, B, 1, dW_out, db_out, G, workspace, p, stream, top_step_done);
}

}  // namespace

extern "C" {

int pfg_version(void) { return 104; }

const char *pfg_last_error(void) { return g_err; }

int pfg_timing_enable(int on) {
  g_timing_on.store(on != 0, std::memory_order_relaxed);
  return PFG_OK;
}

int pfg_timing_reset(void) {
  drain_pending();
  std::lock_guard<std::mutex> lk(g_timing_mu);
  g_totals.clear();
  return PFG_OK;
}

int pfg_timing_query(const char *name, int64_t *launches, double *total_ms) {
  if (!name || !launches || !total_ms) return fail(PFG_ERR_NULL, "pfg_timing_query: NULL argument");
  drain_pending();
  std::lock_guard<std::mutex> lk(g_timing_mu);
  auto it = g_totals.find(name);
  if (it == g_totals.end()) return fail(PFG_ERR_SHAPE, "no launch of '%s' was recorded", name);
  *launches = it->second.first;
  *total_ms = it->second.second;
  return PFG_OK;
}

int pfg_timing_names(char *buf, size_t cap) {
  if (!buf || cap == 0) return fail(PFG_ERR_NULL, "pfg_timing_names: NULL buffer");
  drain_pending();
  std::lock_guard<std::mutex> lk(g_timing_mu);
  std::string s;
  for (auto &kv : g_totals) {
    if (!s.empty()) s += "\n";
    s += kv.first;
  }
  snprintf(buf, cap, "%s", s.c_str());
  return PFG_OK;
}

int pfg_fill_reference(float *out, int64_t n, float value, int stores_per_lane, void *hip_stream) {
  g_err[0] = 0;
  if (!out) return fail(PFG_ERR_NULL, "out is NULL");
  if (n < 0 || (n & 3)) return fail(PFG_ERR_SHAPE, "n = %lld must be a non-negative multiple of 4", (long long)n);
  if (reinterpret_cast<uintptr_t>(out) & 15) return fail(PFG_ERR_SHAPE, "out is not 16-byte aligned");
  if (stores_per_lane != 1 && stores_per_lane != 2 && stores_per_lane != 4 && stores_per_lane != 8 &&
      stores_per_lane != 16)
    return fail(PFG_ERR_UNSUPPORTED, "stores_per_lane = %d is none of 1, 2, 4, 8, 16", stores_per_lane);
  PFG_LAUNCH("fill_reference",
             launch_fill_reference(out, n, value, stores_per_lane, static_cast<hipStream_t>(hip_stream)));
  return PFG_OK;
}

int pfg_workspace_bytes(const pfg_mlp *net, int op, int64_t B, int64_t S, size_t *bytes) {
  g_err[0] = 0;
  int rc = check_net(net);
  if (rc) return rc;
  if (!bytes) return fail(PFG_ERR_NULL, "bytes is NULL");
  if (op < PFG_OP_PER_EXAMPLE_GRADS || op > PFG_OP_HESSIAN_INPUT)
    return fail(PFG_ERR_UNSUPPORTED, "unknown op %d", op);
  if (op == PFG_OP_PER_EXAMPLE_GRADS || op == PFG_OP_GRAD_NORMS) S = 1;
  if ((rc = check_rows(B, S))) return rc;
  if (op == PFG_OP_HESSIAN_INPUT) {
    if ((rc = check_hessian(net, B, S))) return rc;
  } else if ((rc = check_elems(net, B * S))) {
    return rc;
  }
  *bytes = make_plan(net, op, B, S).total;
  return PFG_OK;
}

int pfg_per_example_grads(const pfg_mlp *net, const void *X, const int32_t *labels, int64_t B,
                          float *const *dW_out, float *const *db_out, float *loss_out,
                          void *workspace, size_t workspace_bytes, void *hip_stream) {
  return per_example_grads_impl(net, X, labels, B, dW_out, db_out, loss_out, workspace,
                                workspace_bytes, false, hip_stream);
}

int pfg_per_example_grads_static(const pfg_mlp *net, const void *X, const int32_t *labels, int64_t B,
                                 float *const *dW_out, float *const *db_out, float *loss_out,
                                 void *hip_stream) {
  return per_example_grads_impl(net, X, labels, B, dW_out, db_out, loss_out, nullptr, 0, true,
                                hip_stream);
}

int pfg_per_example_grad_norms(const pfg_mlp *net, const void *X, const int32_t *labels, int64_t B,
                               float *sq_layers_out, float *norm_out, float *loss_out,
                               void *workspace, size_t workspace_bytes, void *hip_stream) {
  g_err[0] = 0;
  int rc = check_net(net);
  if (rc) return rc;
  if ((rc = check_weights(net))) return rc;
  if (!X) return fail(PFG_ERR_NULL, "X is NULL");
  if (!labels) return fail(PFG_ERR_NULL, "labels is NULL");
  if (!sq_layers_out && !norm_out) return fail(PFG_ERR_NULL, "sq_layers_out and norm_out are both NULL");
  if ((rc = check_rows(B, 1))) return rc;
  if ((rc = check_elems(net, B))) return rc;
  const Plan p = make_plan(net, PFG_OP_GRAD_NORMS, B, 1);
  if ((rc = check_workspace(p, workspace, workspace_bytes))) return rc;

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const int L = net->num_layers;
  const int32_t *d = net->dims;

  std::vector<float *> G(L + 1, nullptr);
  for (int l = 1; l <= L; ++l) G[l] = at(workspace, p.G[l]);

  // forward pass and cotangent chain exactly as for the gradients themselves
  bool top_step_done = false;
  if (d[L] <= 32) {
    top_step_done = (L >= 2);
    const HeadFusion hf{labels, G[L], loss_out, top_step_done ? G[L - 1] : nullptr};
    if ((rc = forward(net, X, B, L, workspace, p, true, stream, &hf))) return rc;
  } else {
    if ((rc = forward(net, X, B, L, workspace, p, true, stream))) return rc;
    PFG_LAUNCH("head", launch_head_softmax_ce(at(workspace, p.logits), labels, B, d[L], G[L],
                                              loss_out, stream));
  }
  for (int l = top_step_done ? L - 1 : L; l > 1; --l)
    if ((rc = cotangent_step(net, l, G[l], B, 1, G[l - 1], workspace, p, stream))) return rc;

  // the outer products are never formed: only the squared norms of their two factors
  std::vector<NormLayer> layers(L);
  for (int l = 1; l <= L; ++l) {
    NormLayer &ly = layers[l - 1];
    ly.a = (l == 1) ? X : at(workspace, p.act[l - 1]);
    ly.a_bf16 = (l == 1) && (net->dtype == PFG_BF16);
    ly.g = G[l];
    ly.d_in = d[l - 1];
    ly.d_out = d[l];
    ly.has_bias = (bias_of(net, l) != nullptr);
    ly.index = l - 1;
  }
  if (L <= kNormLayers) {
    PFG_LAUNCH("grad_norms", launch_grad_sqnorms(layers.data(), L, B, sq_layers_out, L, norm_out, stream));
  } else {
    float *sq = sq_layers_out ? sq_layers_out : at(workspace, p.sq);
    for (int l0 = 0; l0 < L; l0 += kNormLayers)
      PFG_LAUNCH("grad_norms", launch_grad_sqnorms(layers.data() + l0, std::min(kNormLayers, L - l0), B,
                                                   sq, L, nullptr, stream));
    if (norm_out) PFG_LAUNCH("grad_norms", launch_norm_finalize(sq, L, L, B, norm_out, stream));
  }
  return PFG_OK;
}

int pfg_hessian_input(const pfg_mlp *net, const void *X, int64_t B, const float *seeds, int64_t S,
                      int64_t seed_batch_stride, float *H_out, void *workspace,
                      size_t workspace_bytes, void *hip_stream) {
  g_err[0] = 0;
  int rc = check_net(net);
  if (rc) return rc;
  if ((rc = check_weights(net))) return rc;
  if (!X) return fail(PFG_ERR_NULL, "X is NULL");
  if (!H_out) return fail(PFG_ERR_NULL, "H_out is NULL");
  if ((rc = check_rows(B, S))) return rc;
  if ((rc = check_seeds(net, seeds, S, seed_batch_stride))) return rc;
  if ((rc = check_hessian(net, B, S))) return rc;
  const Plan p = make_plan(net, PFG_OP_HESSIAN_INPUT, B, S);
  if ((rc = check_workspace(p, workspace, workspace_bytes))) return rc;

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const int L = net->num_layers;
  const int32_t *d = net->dims;
  const int64_t n = d[0], rows = B * S, ktot = p.ktot;
  // a bfloat16 network: its weights (and X) enter the products of the three sweeps as they are, the
  // float32 intermediates are rounded when staged as matrix-core operands; the tangents, cotangents
  // and the final batched product (both operands intermediates) stay float32
  const int32_t bf16 = (net->dtype == PFG_BF16);

  if (L == 1 || net->hidden_act == PFG_ACT_IDENTITY || net->hidden_act == PFG_ACT_RELU) {
    // piecewise-linear network: every second derivative vanishes
    PFG_LAUNCH("fill_zero", launch_fill_zero(H_out, rows * n * n, stream));
    return PFG_OK;
  }
  const int H = L - 1;   // hidden layers 1..H

  // ---- forward pass: z_l, then a_l, phi'(z_l) and phi''(z_l) ----
  for (int l = 1; l <= H; ++l) {
    GemmArgs g{};
    g.A = (l == 1) ? X : at(workspace, p.act[l - 1]);
    g.lda = d[l - 1]; g.a_batch_stride = d[l - 1]; g.S = 1; g.a_is_f32 = (l == 1) ? !bf16 : 1;
    g.W = net->W[l - 1]; g.ldw = d[l]; g.w_kn = 1; g.bf16 = bf16;
    g.M = (int32_t)B; g.N = d[l]; g.K = d[l - 1];
    g.bias = bias_of(net, l);
    g.epilogue = EPI_BIAS;
    g.C = at(workspace, p.d2phi[l]);      // holds z_l until the next kernel overwrites it in place
    g.ldc = d[l];
    PFG_LAUNCH("gemm_forward", launch_gemm(g, stream));
    PFG_LAUNCH("activation", launch_act_from_z(at(workspace, p.d2phi[l]), B, d[l], net->hidden_act,
                                               l < H ? at(workspace, p.act[l]) : nullptr,
                                               at(workspace, p.dphi[l]), at(workspace, p.d2phi[l]),
                                               stream));
  }

  // ---- tangents: U_l[b] = (d z_l[b] / d x_b)^T, [d_0, d_l], side by side in U [B * d_0, ktot] ----
  // U_1 = W_1 for every b; U_{l+1}[b] = (U_l[b] * phi'(z_l[b, :])) W_{l+1}: rows (b, i) folded into
  // one product with the loop-invariant W_{l+1}, the mask broadcast over i.
  float *U = at(workspace, p.U);
  PFG_LAUNCH("tangent_seed", launch_scale_rows(net->W[0], bf16, 0, d[1], nullptr, 0, B, n, d[1], U, ktot,
                                               stream));
  for (int l = 1; l < H; ++l) {
    GemmArgs g{};
    g.A = U + p.koff[l]; g.lda = ktot; g.a_batch_stride = n * ktot; g.S = (int32_t)n; g.a_is_f32 = 1;
    g.a_scale = at(workspace, p.dphi[l]); g.ld_scale = d[l];
    g.W = net->W[l]; g.ldw = d[l + 1]; g.w_kn = 1; g.bf16 = bf16;
    g.M = (int32_t)(B * n); g.N = d[l + 1]; g.K = d[l];
    g.epilogue = EPI_NONE;
    g.C = U + p.koff[l + 1]; g.ldc = ktot;
    PFG_LAUNCH("gemm_tangent", launch_gemm(g, stream));
  }

  // ---- cotangents at a_l (before the mask), times phi''(z_l): Cc [B * S, ktot] ----
  float *Cc = at(workspace, p.Cc);
  float *bufs[2] = {at(workspace, p.ping), at(workspace, p.pong)};
  int which = 0;
  const float *cur;
  int64_t cur_bstride;
  const bool shared = (seeds == nullptr) || (seed_batch_stride == 0);
  {
    GemmArgs g{};
    g.A = seeds; g.lda = d[L]; g.S = (int32_t)S; g.a_is_f32 = 1;
    g.W = net->W[L - 1]; g.ldw = d[L]; g.w_kn = 0; g.bf16 = bf16;
    g.N = d[H]; g.K = d[L];
    g.epilogue = EPI_NONE; g.ldc = d[H];
    if (shared) {
      // loop-invariant seeds: the product does not depend on b and is formed once, not stacked
      float *P = at(workspace, p.P);
      if (!seeds) {
        PFG_LAUNCH("transpose", launch_transpose(net->W[L - 1], bf16, d[H], d[L], P, stream));
      } else {
        g.a_batch_stride = 0; g.M = (int32_t)S; g.C = P;
        PFG_LAUNCH("gemm_cotangent", launch_gemm(g, stream));
      }
      cur = P; cur_bstride = 0;
    } else {
      g.a_batch_stride = seed_batch_stride; g.M = (int32_t)rows; g.C = bufs[which];
      PFG_LAUNCH("gemm_cotangent", launch_gemm(g, stream));
      cur = bufs[which]; cur_bstride = S * d[H];
      which ^= 1;
    }
  }
  for (int l = H; l >= 1; --l) {
    // cur = h_l (cotangent at a_l), rows (b, s)
    PFG_LAUNCH("curvature_rows", launch_scale_rows(cur, 0, cur_bstride, d[l], at(workspace, p.d2phi[l]),
                                                   d[l], B, S, d[l], Cc + p.koff[l], ktot, stream));
    if (l == 1) break;
    GemmArgs g{};
    g.A = cur; g.lda = d[l]; g.a_batch_stride = cur_bstride; g.S = (int32_t)S; g.a_is_f32 = 1;
    g.a_scale = at(workspace, p.dphi[l]); g.ld_scale = d[l];
    g.W = net->W[l - 1]; g.ldw = d[l]; g.w_kn = 0; g.bf16 = bf16;
    g.M = (int32_t)rows; g.N = d[l - 1]; g.K = d[l];
    g.epilogue = EPI_NONE;
    g.C = bufs[which]; g.ldc = d[l - 1];
    PFG_LAUNCH("gemm_cotangent", launch_gemm(g, stream));
    cur = bufs[which]; cur_bstride = S * d[l - 1];
    which ^= 1;
  }

  // ---- H[b, (s, i), j] = sum_k U[b, i, k] Cc[b, s, k] U[b, j, k]: one product per example, both
  // operands stacked (Section 3.4's batched matmul); the weights Cc scale the A rows as they are staged ----
  for (int64_t b0 = 0; b0 < B; b0 += 32768) {
    const int64_t nb = std::min<int64_t>(32768, B - b0);
    GemmArgs g{};
    g.A = U + b0 * n * ktot; g.lda = ktot; g.a_batch_stride = 0; g.S = (int32_t)n; g.a_is_f32 = 1;
    g.a_scale = Cc + b0 * S * ktot; g.ld_scale = ktot;
    g.W = U + b0 * n * ktot; g.ldw = ktot; g.w_kn = 0;
    g.M = (int32_t)(S * n); g.N = (int32_t)n; g.K = (int32_t)ktot;
    g.epilogue = EPI_NONE;
    g.C = H_out + b0 * S * n * n; g.ldc = n;
    g.streaming = 1;
    g.nbatch = (int32_t)nb;
    g.batch_A = n * ktot; g.batch_scale = S * ktot; g.batch_W = n * ktot; g.batch_C = S * n * n;
    // second derivatives commute: each H[b, s] is symmetric, so the tiles below its diagonal are
    // mirror images of those above and need not be computed
    if (n % 128 == 0) g.sym_n = (int32_t)n;
    PFG_LAUNCH("gemm_hessian", launch_gemm(g, stream));
  }
  return PFG_OK;
}

}  // extern "C"

namespace {

struct ConvBlock {
  int h, w, ci, co, k;     // input size and channels, output channels, kernel size
  size_t P, PT, z, pooled, which, dz;
  size_t gW = 0, gb = 0;   // norms only: this block's per-example filter and bias gradients
};

struct ConvPlan {
  size_t total = 0;
  std::vector<ConvBlock> blocks;
  size_t dout[2] = {0, 0};     // cotangents of pooled outputs, used alternately
  size_t psum = 0;             // partial sums over positions (bias gradients)
  size_t dense = 0;            // sub-workspace of the dense layers
  size_t dense_bytes = 0;
  size_t sq = 0;               // norms only: [B, num_conv + L] squared norms when the caller wants none
  size_t take(size_t bytes) {
    const size_t at = total;
    total += (bytes + 255) / 256 * 256;
    return at;
  }
};

int check_convnet(const pfg_convnet *net, int64_t B) {
  if (!net) return fail(PFG_ERR_NULL, "net is NULL");
  if (net->num_conv < 1 || net->num_conv > 64)
    return fail(PFG_ERR_SHAPE, "num_conv = %d is outside [1, 64]", net->num_conv);
  if (!net->kernel || !net->filters) return fail(PFG_ERR_NULL, "net->kernel or net->filters is NULL");
  if (net->height < 1 || net->width < 1 || net->channels < 1)
    return fail(PFG_ERR_SHAPE, "image size %d x %d x %d", net->height, net->width, net->channels);
  int rc = check_net(&net->dense);
  if (rc) return rc;
  if (net->dense.dtype != PFG_F32)
    return fail(PFG_ERR_UNSUPPORTED, "the convolutional path is float32 only (dtype %d given)", net->dense.dtype);
  if (B < 1 || B > 65535) return fail(PFG_ERR_SHAPE, "B = %lld is outside [1, 65535]", (long long)B);
  int64_t h = net->height, w = net->width, c = net->channels;
  for (int i = 0; i < net->num_conv; ++i) {
    const int64_t k = net->kernel[i], f = net->filters[i];
    if (k < 1 || k % 2 == 0 || k > 31) return fail(PFG_ERR_SHAPE, "kernel[%d] = %lld must be odd and at most 31", i, (long long)k);
    if (f < 1 || f > (1 << 16)) return fail(PFG_ERR_SHAPE, "filters[%d] = %lld is out of range", i, (long long)f);
    if (h % 2 || w % 2) return fail(PFG_ERR_SHAPE, "conv block %d sees a %lld x %lld image; both must be even", i, (long long)h, (long long)w);
    if (h * w * k * k * c > 0x7fffffffLL / 2 || B * h * w > kMaxRows || B * h * w * k * k * c > kMaxElems)
      return fail(PFG_ERR_OVERFLOW, "conv block %d is too large for B = %lld", i, (long long)B);
    h /= 2; w /= 2; c = f;
  }
  if (h * w * c != net->dense.dims[0])
    return fail(PFG_ERR_SHAPE, "the conv blocks produce %lld features, dense.dims[0] is %d", (long long)(h * w * c), net->dense.dims[0]);
  return PFG_OK;
}

ConvPlan make_conv_plan(const pfg_convnet *net, int64_t B, bool norms = false) {
  ConvPlan p;
  const size_t f = sizeof(float);
  int h = net->height, w = net->width, c = net->channels;
  size_t widest_pooled = 0;
  for (int i = 0; i < net->num_conv; ++i) {
    ConvBlock blk{};
    blk.h = h; blk.w = w; blk.ci = c; blk.co = net->filters[i]; blk.k = net->kernel[i];
    const size_t hw = (size_t)h * w, kkc = (size_t)blk.k * blk.k * c, cells = (size_t)(h / 2) * (w / 2) * blk.co;
    blk.P = p.take(f * B * hw * kkc);
    blk.PT = p.take(f * B * hw * kkc);
    blk.z = p.take(f * B * hw * blk.co);
    blk.dz = p.take(f * B * hw * blk.co);
    blk.pooled = p.take(f * B * cells);
    blk.which = p.take(B * cells);
    widest_pooled = std::max(widest_pooled, B * cells);
    if (norms) {
      blk.gW = p.take(f * B * kkc * blk.co);
      blk.gb = p.take(f * B * blk.co);
    }
    p.blocks.push_back(blk);
    h /= 2; w /= 2; c = blk.co;
  }
  p.dout[0] = p.take(f * widest_pooled);
  p.dout[1] = p.take(f * widest_pooled);
  size_t widest_co = 0;
  for (const ConvBlock &blk : p.blocks) widest_co = std::max(widest_co, (size_t)blk.co);
  p.psum = p.take(f * B * kSumPieces * widest_co);
  p.dense_bytes = make_plan(&net->dense, PFG_OP_PER_EXAMPLE_GRADS, B, 1).total;
  p.dense = p.take(p.dense_bytes);
  if (norms) p.sq = p.take(f * B * (net->num_conv + net->dense.num_layers));
  return p;
}

// The squared norms wanted from the sweep instead of the gradients themselves.
struct ConvNorms {
  float *sq_blocks;   // [B, num_conv + L] or null
  float *norm;        // [B] or null
};

int check_convnet_call(const pfg_convnet *net, const void *X, const int32_t *labels, int64_t B,
                       const ConvPlan &cp, void *workspace, size_t workspace_bytes) {
  int rc = check_weights(&net->dense);
  if (rc) return rc;
  if (!net->Wc) return fail(PFG_ERR_NULL, "net->Wc is NULL");
  for (int i = 0; i < net->num_conv; ++i)
    if (!net->Wc[i]) return fail(PFG_ERR_NULL, "net->Wc[%d] is NULL", i);
  if (!X) return fail(PFG_ERR_NULL, "X is NULL");
  if (!labels) return fail(PFG_ERR_NULL, "labels is NULL");
  if (!workspace) return fail(PFG_ERR_WORKSPACE, "workspace is NULL (%zu bytes needed)", cp.total);
  if (reinterpret_cast<uintptr_t>(workspace) & 255) return fail(PFG_ERR_WORKSPACE, "workspace is not 256-byte aligned");
  if (workspace_bytes < cp.total)
    return fail(PFG_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, cp.total);
  return PFG_OK;
}

// A filter gradient of one example must fit a row index of the norm kernel and the scratch block
// of all examples the element limit of the products.
int check_convnet_norms(const pfg_convnet *net, int64_t B) {
  int64_t c = net->channels;
  for (int i = 0; i < net->num_conv; ++i) {
    const int64_t k = net->kernel[i], f = net->filters[i];
    if (k * k * c * f > 0x7fffffffLL || B * k * k * c * f > kMaxElems)
      return fail(PFG_ERR_OVERFLOW, "the filter gradients of conv block %d are too large for B = %lld", i, (long long)B);
    c = f;
  }
  return PFG_OK;
}

int convnet_sweep(const pfg_convnet *net, const void *X, const int32_t *labels, int64_t B,
                  float *const *dWc_out, float *const *dbc_out, float *const *dW_out,
                  float *const *db_out, float *loss_out, const ConvNorms *norms, const ConvPlan &cp,
                  void *workspace, hipStream_t stream);

}  // namespace

extern "C" {

int pfg_convnet_workspace_bytes(const pfg_convnet *net, int64_t B, size_t *bytes) {
  g_err[0] = 0;
  int rc = check_convnet(net, B);
  if (rc) return rc;
  if (!bytes) return fail(PFG_ERR_NULL, "bytes is NULL");
  if ((rc = check_elems(&net->dense, B))) return rc;
  *bytes = make_conv_plan(net, B).total;
  return PFG_OK;
}

int pfg_convnet_per_example_grads(const pfg_convnet *net, const void *X, const int32_t *labels,
                                  int64_t B, float *const *dWc_out, float *const *dbc_out,
                                  float *const *dW_out, float *const *db_out, float *loss_out,
                                  void *workspace, size_t workspace_bytes, void *hip_stream) {
  g_err[0] = 0;
  int rc = check_convnet(net, B);
  if (rc) return rc;
  if ((rc = check_elems(&net->dense, B))) return rc;
  const ConvPlan cp = make_conv_plan(net, B);
  if ((rc = check_convnet_call(net, X, labels, B, cp, workspace, workspace_bytes))) return rc;
  return convnet_sweep(net, X, labels, B, dWc_out, dbc_out, dW_out, db_out, loss_out, nullptr, cp,
                       workspace, static_cast<hipStream_t>(hip_stream));
}

int pfg_convnet_grad_norms_workspace_bytes(const pfg_convnet *net, int64_t B, size_t *bytes) {
  g_err[0] = 0;
  int rc = check_convnet(net, B);
  if (rc) return rc;
  if (!bytes) return fail(PFG_ERR_NULL, "bytes is NULL");
  if ((rc = check_elems(&net->dense, B))) return rc;
  if ((rc = check_convnet_norms(net, B))) return rc;
  *bytes = make_conv_plan(net, B, true).total;
  return PFG_OK;
}

int pfg_convnet_per_example_grad_norms(const pfg_convnet *net, const void *X, const int32_t *labels,
                                       int64_t B, float *sq_blocks_out, float *norm_out,
                                       float *loss_out, void *workspace, size_t workspace_bytes,
                                       void *hip_stream) {
  g_err[0] = 0;
  int rc = check_convnet(net, B);
  if (rc) return rc;
  if ((rc = check_elems(&net->dense, B))) return rc;
  if ((rc = check_convnet_norms(net, B))) return rc;
  if (!sq_blocks_out && !norm_out) return fail(PFG_ERR_NULL, "sq_blocks_out and norm_out are both NULL");
  const ConvPlan cp = make_conv_plan(net, B, true);
  if ((rc = check_convnet_call(net, X, labels, B, cp, workspace, workspace_bytes))) return rc;
  // the filter and bias gradients go to the workspace; only their squared sums leave it
  const int nc = net->num_conv;
  std::vector<float *> gW(nc), gb(nc);
  for (int i = 0; i < nc; ++i) {
    gW[i] = at(workspace, cp.blocks[i].gW);
    gb[i] = (net->bc && net->bc[i]) ? at(workspace, cp.blocks[i].gb) : nullptr;
  }
  const ConvNorms norms{sq_blocks_out, norm_out};
  return convnet_sweep(net, X, labels, B, gW.data(), gb.data(), nullptr, nullptr, loss_out, &norms, cp,
                       workspace, static_cast<hipStream_t>(hip_stream));
}

}  // extern "C"

namespace {

int convnet_sweep(const pfg_convnet *net, const void *X, const int32_t *labels, int64_t B,
                  float *const *dWc_out, float *const *dbc_out, float *const *dW_out,
                  float *const *db_out, float *loss_out, const ConvNorms *norms, const ConvPlan &cp,
                  void *workspace, hipStream_t stream) {
  int rc = PFG_OK;
  void *ws = workspace;
  const pfg_mlp *dn = &net->dense;
  const int L = dn->num_layers, nc = net->num_conv;
  const int32_t *d = dn->dims;

  // The per-example filter gradient of block i: both operands stacked (Section 3.4), for each
  // example [k k c_in, h w] x [h w, c_out].  Its A operand is the example's patch matrix with the
  // POSITION as the contraction index.  The product reads the position-major patches P as a
  // transposed operand when it can (transposed = true); otherwise it needs the second copy PT with
  // the position index fastest, which the forward pass then has to write.
  auto filter_product = [&](int i, bool transposed) {
    const ConvBlock &blk = cp.blocks[i];
    const int hw = blk.h * blk.w, kkc = blk.k * blk.k * blk.ci;
    GemmArgs g{};
    if (transposed) {
      g.A = at(ws, blk.P); g.a_km = 1; g.lda = kkc; g.S = 1;
    } else {
      g.A = at(ws, blk.PT); g.lda = hw; g.a_batch_stride = 0; g.S = kkc;
    }
    g.a_is_f32 = 1;
    g.W = at(ws, blk.dz); g.ldw = blk.co; g.w_kn = 1;
    g.M = kkc; g.N = blk.co; g.K = hw;
    g.epilogue = EPI_NONE;
    g.C = dWc_out[i]; g.ldc = blk.co; g.streaming = norms ? 0 : 1;   // the norm kernel reads it back
    g.nbatch = (int32_t)B;
    g.batch_A = (int64_t)kkc * hw; g.batch_W = (int64_t)hw * blk.co; g.batch_C = (int64_t)kkc * blk.co;
    return g;
  };
  auto filter_reads_P = [&](int i) {
    const GemmArgs g = filter_product(i, true);
    return g.K % 4 == 0 && akm_supported(g);
  };
  // The input image of every block (X, then the pooled outputs), and whether the block's products
  // gather their patches from it themselves: the forward product over the rows (b, y, x) and the
  // filter-gradient product over the positions then need no patch matrix at all (channel counts
  // that are multiples of 4, enough tiles for the tiled kernel).
  std::vector<const float *> image(nc);
  auto forward_product = [&](int i, bool gathered) {
    const ConvBlock &blk = cp.blocks[i];
    const int kkc = blk.k * blk.k * blk.ci;
    GemmArgs g{};
    if (gathered) {
      g.A = image[i]; g.conv_k = blk.k; g.conv_h = blk.h; g.conv_w = blk.w; g.conv_c = blk.ci;
    } else {
      g.A = at(ws, blk.P);
    }
    g.lda = kkc; g.a_batch_stride = kkc; g.S = 1; g.a_is_f32 = 1;
    g.W = net->Wc[i]; g.ldw = blk.co; g.w_kn = 1;
    g.M = (int32_t)(B * blk.h * blk.w); g.N = blk.co; g.K = kkc;
    g.bias = net->bc ? net->bc[i] : nullptr;
    g.epilogue = EPI_BIAS;
    g.C = at(ws, blk.z); g.ldc = blk.co;
    return g;
  };
  auto gathered_filter_product = [&](int i) {
    const ConvBlock &blk = cp.blocks[i];
    GemmArgs g = filter_product(i, true);
    g.A = image[i]; g.conv_k = blk.k; g.conv_h = blk.h; g.conv_w = blk.w; g.conv_c = blk.ci;
    g.batch_A = (int64_t)blk.h * blk.w * blk.ci;
    return g;
  };
  auto gathers = [&](int i) {
    const ConvBlock &blk = cp.blocks[i];
    if (blk.ci % 4 != 0 || image[i] == nullptr) return false;
    const int64_t tiles = ((B * blk.h * blk.w + 63) / 64) * ((blk.co + 63) / 64);
    return tiles >= 128 && conv_gather_supported(forward_product(i, true)) &&
           conv_gather_supported(gathered_filter_product(i));
  };

  // ---- conv blocks, forward: patches, one product over the rows (b, y, x), relu + pooling ----
  const float *in = static_cast<const float *>(X);
  for (int i = 0; i < nc; ++i) {
    const ConvBlock &blk = cp.blocks[i];
    image[i] = in;
    const bool want_filter = dWc_out && dWc_out[i];
    const bool gathered = gathers(i);
    uint8_t *which = reinterpret_cast<uint8_t *>(static_cast<char *>(ws) + blk.which);
    const float *bias = net->bc ? static_cast<const float *>(net->bc[i]) : nullptr;
    const float *filt = static_cast<const float *>(net->Wc[i]);
    // few taps per output: one kernel from the image to the pooled output, and patches only for
    // the filter gradient, in the layout that product reads
    const bool direct = conv_relu_pool_applies(in, filt, bias, B, blk.h, blk.w, blk.ci, blk.k, blk.co,
                                               at(ws, blk.pooled), which);
    // many channels on a small map: the matrix-core kernels that read the image from LDS in place
    const bool direct_mfma = !direct && conv_direct_forward_applies(in, filt, bias, B, blk.h, blk.w, blk.ci, blk.k,
                                                                    blk.co, at(ws, blk.pooled), which);
    const bool filter_direct = want_filter &&
        (conv_filter_direct_applies(in, at(ws, blk.dz), B, blk.h, blk.w, blk.ci, blk.k, blk.co, dWc_out[i]) ||
         conv_filter_rows_applies(in, at(ws, blk.dz), B, blk.h, blk.w, blk.ci, blk.k, blk.co, dWc_out[i]));
    const bool filter_P = want_filter && !filter_direct && !gathered && filter_reads_P(i);
    const bool filter_PT = want_filter && !filter_direct && !gathered && !filter_reads_P(i);
    const bool forward_P = !gathered && !direct && !direct_mfma;
    if (forward_P || filter_P || filter_PT)
      PFG_LAUNCH("im2col", launch_im2col(in, B, blk.h, blk.w, blk.ci, blk.k,
                                         (forward_P || filter_P) ? at(ws, blk.P) : nullptr,
                                         filter_PT ? at(ws, blk.PT) : nullptr, stream));
    if (direct) {
      PFG_LAUNCH("conv_relu_pool", launch_conv_relu_pool(in, filt, bias, B, blk.h, blk.w, blk.ci, blk.k,
                                                         blk.co, at(ws, blk.pooled), which, stream));
    } else if (direct_mfma) {
      PFG_LAUNCH("conv_gemm_forward", launch_conv_direct_forward(in, filt, bias, B, blk.h, blk.w, blk.ci, blk.k,
                                                                 blk.co, at(ws, blk.pooled), which, stream));
    } else {
      PFG_LAUNCH("conv_gemm_forward", launch_gemm(forward_product(i, gathered), stream));
      PFG_LAUNCH("relu_pool", launch_relu_pool(at(ws, blk.z), B, blk.h, blk.w, blk.co, at(ws, blk.pooled), which,
                                               stream));
    }
    in = at(ws, blk.pooled);
  }
  const float *feat = in;       // [B, d_0]

  // ---- dense layers: forward, loss head, cotangent chain down to layer 1 ----
  void *dws = static_cast<char *>(ws) + cp.dense;
  const Plan p = make_plan(dn, PFG_OP_PER_EXAMPLE_GRADS, B, 1);
  std::vector<float *> G(L + 1, nullptr);
  for (int l = 1; l <= L; ++l) G[l] = (db_out && db_out[l - 1]) ? db_out[l - 1] : at(dws, p.G[l]);
  bool top_step_done = false;
  if (d[L] <= 32) {
    top_step_done = (L >= 2);
    const HeadFusion hf{labels, G[L], loss_out, top_step_done ? G[L - 1] : nullptr};
    if ((rc = forward(dn, feat, B, L, dws, p, true, stream, &hf))) return rc;
  } else {
    if ((rc = forward(dn, feat, B, L, dws, p, true, stream))) return rc;
    PFG_LAUNCH("head", launch_head_softmax_ce(at(dws, p.logits), labels, B, d[L], G[L], loss_out, stream));
  }
  for (int l = top_step_done ? L - 1 : L; l > 1; --l)
    if ((rc = cotangent_step(dn, l, G[l], B, 1, G[l - 1], dws, p, stream))) return rc;
  {
    std::vector<OuterArgs> jobs;
    for (int l = 1; l <= L; ++l)
      if (dW_out && dW_out[l - 1]) jobs.push_back(outer_job(dn, l, feat, G[l], B, 1, dW_out[l - 1], dws, p));
    std::stable_sort(jobs.begin(), jobs.end(), [](const OuterArgs &x, const OuterArgs &y) {
      return (int64_t)x.d_in * x.d_out > (int64_t)y.d_in * y.d_out;
    });
    if (!jobs.empty()) PFG_LAUNCH("outer_product", launch_outer(jobs.data(), (int)jobs.size(), stream));
  }
  bool any_conv = false;
  for (int i = 0; i < nc; ++i) any_conv = any_conv || (dWc_out && dWc_out[i]) || (dbc_out && dbc_out[i]);
  if (!any_conv) return PFG_OK;

  // cotangent of the flattened features: G_1 W_1^T (nothing masks it: the pooling step follows)
  float *dout = at(ws, cp.dout[0]);
  int which_dout = 0;
  {
    GemmArgs g{};
    g.A = G[1]; g.lda = d[1]; g.a_batch_stride = d[1]; g.S = 1; g.a_is_f32 = 1;
    g.W = dn->W[0]; g.ldw = d[1]; g.w_kn = 0;
    g.M = (int32_t)B; g.N = d[0]; g.K = d[1];
    g.epilogue = EPI_NONE; g.C = dout; g.ldc = d[0];
    PFG_LAUNCH("gemm_cotangent", launch_gemm(g, stream));
  }

  // ---- conv blocks, reverse ----
  std::vector<int> sq_parts(nc, 0);     // > 0: the block's filter gradient left that many partial sums of squares
  for (int i = nc - 1; i >= 0; --i) {
    const ConvBlock &blk = cp.blocks[i];
    const int hw = blk.h * blk.w, kkc = blk.k * blk.k * blk.ci;
    const int64_t rows = B * hw;
    float *dz = at(ws, blk.dz);
    const uint8_t *which = reinterpret_cast<const uint8_t *>(static_cast<char *>(ws) + blk.which);
    float *dbc = dbc_out ? dbc_out[i] : nullptr;
    if (dbc && unpool_mask_sum_applies(dout, at(ws, blk.pooled), which, B, blk.h, blk.w, blk.co, dz, dbc)) {
      PFG_LAUNCH("unpool_mask", launch_unpool_mask_sum(dout, at(ws, blk.pooled), which, B, blk.h, blk.w,
                                                     blk.co, dz, dbc, stream));
    } else {
      PFG_LAUNCH("unpool_mask", launch_unpool_mask(dout, at(ws, blk.pooled), which, B, blk.h, blk.w, blk.co,
                                                   dz, stream));
      if (dbc) PFG_LAUNCH("sum_positions", launch_sum_steps(dz, B, hw, blk.co, dbc, at(ws, cp.psum), stream));
    }
    if (dWc_out && dWc_out[i]) {
      // when only norms are wanted, the kernels that form the gradient on the LDS image store the sums
      // of its squares (a few per example, at the head of the buffer meant for the gradient) and no gradient
      float *sq_part = norms ? dWc_out[i] : nullptr;
      if (conv_filter_direct_applies(image[i], dz, B, blk.h, blk.w, blk.ci, blk.k, blk.co, dWc_out[i])) {
        PFG_LAUNCH("conv_gemm_filter", launch_conv_filter_direct(image[i], dz, B, blk.h, blk.w, blk.ci, blk.k,
                                                                 blk.co, dWc_out[i], 1, sq_part, stream));
        if (norms) sq_parts[i] = conv_filter_direct_parts(blk.ci, blk.co);
      } else if (conv_filter_rows_applies(image[i], dz, B, blk.h, blk.w, blk.ci, blk.k, blk.co, dWc_out[i])) {
        PFG_LAUNCH("conv_gemm_filter", launch_conv_filter_rows(image[i], dz, B, blk.h, blk.w, blk.ci, blk.k, blk.co,
                                                               dWc_out[i], 1, sq_part, stream));
        if (norms) sq_parts[i] = conv_filter_rows_parts(blk.co);
      }
      else
        PFG_LAUNCH("conv_gemm_filter", launch_gemm(gathers(i) ? gathered_filter_product(i)
                                                              : filter_product(i, filter_reads_P(i)), stream));
    }
    bool lower = false;
    for (int j = 0; j < i; ++j) lower = lower || (dWc_out && dWc_out[j]) || (dbc_out && dbc_out[j]);
    if (!lower) break;
    // the same matrix-core kernel as the forward pass, run on dz with the filter flipped and transposed
    if (conv_direct_reverse_applies(dz, static_cast<const float *>(net->Wc[i]), B, blk.h, blk.w, blk.ci, blk.k,
                                    blk.co, at(ws, cp.dout[which_dout ^ 1]))) {
      which_dout ^= 1;
      dout = at(ws, cp.dout[which_dout]);
      PFG_LAUNCH("conv_gemm_cotangent", launch_conv_direct_reverse(dz, static_cast<const float *>(net->Wc[i]), B,
                                                                   blk.h, blk.w, blk.ci, blk.k, blk.co, dout, stream));
      continue;
    }
    // cotangent of the patches, dP = dz Wc^T (into the patch buffer, no longer needed), gathered
    // back to the image that entered this block = the pooled output of the block below
    GemmArgs g{};
    g.A = dz; g.lda = blk.co; g.a_batch_stride = blk.co; g.S = 1; g.a_is_f32 = 1;
    g.W = net->Wc[i]; g.ldw = blk.co; g.w_kn = 0;
    g.M = (int32_t)rows; g.N = kkc; g.K = blk.co;
    g.epilogue = EPI_NONE; g.C = at(ws, blk.P); g.ldc = kkc;
    PFG_LAUNCH("conv_gemm_cotangent", launch_gemm(g, stream));
    which_dout ^= 1;
    dout = at(ws, cp.dout[which_dout]);
    PFG_LAUNCH("col2im", launch_col2im(at(ws, blk.P), B, blk.h, blk.w, blk.ci, blk.k, dout, stream));
  }
  if (!norms) return PFG_OK;

  // ---- squared norms: a conv block's is the sum of squares of the filter and bias gradients
  // formed above; a dense layer's comes from its two factors, the outer product never formed ----
  const int cols = nc + L;
  std::vector<NormLayer> layers(cols);
  for (int i = 0; i < nc; ++i) {
    const ConvBlock &blk = cp.blocks[i];
    NormLayer &ly = layers[i];
    ly.a = dWc_out[i];
    ly.g = dbc_out[i];             // null for a block without a bias
    ly.d_in = sq_parts[i] ? sq_parts[i] : blk.k * blk.k * blk.ci * blk.co;
    ly.d_out = blk.co;
    ly.sum_mode = sq_parts[i] ? 2 : 1;
    ly.index = i;
  }
  for (int l = 1; l <= L; ++l) {
    NormLayer &ly = layers[nc + l - 1];
    ly.a = (l == 1) ? feat : at(dws, p.act[l - 1]);
    ly.g = G[l];
    ly.d_in = d[l - 1];
    ly.d_out = d[l];
    ly.has_bias = (bias_of(dn, l) != nullptr);
    ly.index = nc + l - 1;
  }
  if (cols <= kNormLayers) {
    PFG_LAUNCH("grad_norms", launch_grad_sqnorms(layers.data(), cols, B, norms->sq_blocks, cols, norms->norm, stream));
  } else {
    float *sq = norms->sq_blocks ? norms->sq_blocks : at(ws, cp.sq);
    for (int l0 = 0; l0 < cols; l0 += kNormLayers)
      PFG_LAUNCH("grad_norms", launch_grad_sqnorms(layers.data() + l0, std::min(kNormLayers, cols - l0), B,
                                                   sq, cols, nullptr, stream));
    if (norms->norm) PFG_LAUNCH("grad_norms", launch_norm_finalize(sq, cols, cols, B, norms->norm, stream));
  }
  return PFG_OK;
}

}  // namespace

extern "C" {

int pfg_jacobian_input(const pfg_mlp *net, const void *X, int64_t B, const float *seeds, int64_t S,
                       int64_t seed_batch_stride, float *J_out, void *workspace,
                       size_t workspace_bytes, void *hip_stream) {
  g_err[0] = 0;
  int rc = check_net(net);
  if (rc) return rc;
  if ((rc = check_weights(net))) return rc;
  if (!X) return fail(PFG_ERR_NULL, "X is NULL");
  if (!J_out) return fail(PFG_ERR_NULL, "J_out is NULL");
  if ((rc = check_rows(B, S))) return rc;
  if ((rc = check_seeds(net, seeds, S, seed_batch_stride))) return rc;
  if ((rc = check_elems(net, B * S))) return rc;
  const Plan p = make_plan(net, PFG_OP_JACOBIAN_INPUT, B, S);
  if ((rc = check_workspace(p, workspace, workspace_bytes))) return rc;

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const int L = net->num_layers;
  const int32_t *d = net->dims;
  const bool bf16 = (net->dtype == PFG_BF16);
  const int64_t rows = B * S;

  // the logits themselves are not needed: the Jacobian depends on phi'(z_l), l < L, only
  if ((rc = forward(net, X, B, L - 1, workspace, p, false, stream))) return rc;

  // Current cotangent block: rows (b, s) at cur + b * cur_bstride + s * cur_ld, times an optional
  // pending mask row b of cur_scale (the mask is invariant over s and is applied while the block
  // is staged as the A operand of the next product).
  const float *cur = seeds;
  int64_t cur_ld = d[L], cur_bstride = seed_batch_stride;
  const float *cur_scale = nullptr;
  int64_t cur_scale_ld = 0;
  int level = L;     // cur is the cotangent at the output of layer `level`
  float *bufs[2] = {at(workspace, p.ping), at(workspace, p.pong)};
  int which = 0;

  const bool shared = (seeds == nullptr) || (seed_batch_stride == 0);
  if (shared && L >= 2) {
    // Loop-invariant seeds: G_{L-1}[b, s, :] = (seeds[s, :] W_L^T) * phi'(z_{L-1}[b, :]).  The
    // product in brackets does not depend on b, so it is formed once ([S, d_{L-1}], not stacked)
    // and the mask is left pending.  Identity seeds make it a transpose of W_L.
    float *P = at(workspace, p.P);
    if (!seeds) {
      PFG_LAUNCH("transpose", launch_transpose(net->W[L - 1], bf16, d[L - 1], d[L], P, stream));
    } else {
      GemmArgs g{};
      g.A = seeds; g.lda = d[L]; g.a_batch_stride = 0; g.S = (int32_t)S; g.a_is_f32 = 1;
      g.W = net->W[L - 1]; g.ldw = d[L]; g.w_kn = 0; g.bf16 = bf16;
      g.M = (int32_t)S; g.N = d[L - 1]; g.K = d[L];
      g.epilogue = EPI_NONE; g.C = P; g.ldc = d[L - 1];
      PFG_LAUNCH("gemm_cotangent", launch_gemm(g, stream));
    }
    cur = P; cur_ld = d[L - 1]; cur_bstride = 0;
    cur_scale = at(workspace, p.dphi[L - 1]); cur_scale_ld = d[L - 1];
    level = L - 1;
  }

  for (int l = level; l >= 1; --l) {
    GemmArgs g{};
    g.S = (int32_t)S;
    g.a_is_f32 = 1;
    g.a_scale = cur_scale; g.ld_scale = cur_scale_ld;
    g.W = net->W[l - 1]; g.ldw = d[l]; g.w_kn = 0; g.bf16 = bf16;
    g.M = (int32_t)rows; g.N = d[l - 1]; g.K = d[l];
    if (cur == nullptr) {
      // identity seeds of a one-layer network: J[b] = W_1^T for every b
      float *P = at(workspace, p.P);
      PFG_LAUNCH("seed_rows", launch_seed_rows(nullptr, nullptr, 0, 1, S, d[L], 0, P, stream));
      cur = P; cur_ld = d[L]; cur_bstride = 0;
    }
    g.A = cur; g.lda = cur_ld; g.a_batch_stride = cur_bstride;
    if (l > 1) {
      g.epilogue = EPI_MASK;
      g.emask = at(workspace, p.dphi[l - 1]); g.ld_emask = d[l - 1];
      g.C = bufs[which]; g.ldc = d[l - 1];
      PFG_LAUNCH("gemm_cotangent", launch_gemm(g, stream));
      cur = bufs[which]; cur_ld = d[l - 1]; cur_bstride = S * d[l - 1];
      cur_scale = nullptr; cur_scale_ld = 0;
      which ^= 1;
    } else {
      g.epilogue = EPI_NONE;
      g.C = J_out; g.ldc = d[0];
      g.streaming = 1;
      PFG_LAUNCH("gemm_jacobian", launch_gemm(g, stream));
    }
  }
  return PFG_OK;
}

int pfg_jacobian_weights(const pfg_mlp *net, const void *X, int64_t B, int head, const float *seeds,
                         int64_t S, int64_t seed_batch_stride, float *const *JW_out,
                         float *const *Jb_out, void *workspace, size_t workspace_bytes,
                         void *hip_stream) {
  g_err[0] = 0;
  int rc = check_net(net);
  if (rc) return rc;
  if ((rc = check_weights(net))) return rc;
  if (!X) return fail(PFG_ERR_NULL, "X is NULL");
  if (head != PFG_HEAD_LOGITS && head != PFG_HEAD_SOFTMAX)
    return fail(PFG_ERR_UNSUPPORTED, "unknown head %d", head);
  if ((rc = check_rows(B, S))) return rc;
  if ((rc = check_seeds(net, seeds, S, seed_batch_stride))) return rc;
  if ((rc = check_elems(net, B * S))) return rc;
  const Plan p = make_plan(net, PFG_OP_JACOBIAN_WEIGHTS, B, S);
  if ((rc = check_workspace(p, workspace, workspace_bytes))) return rc;

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const int L = net->num_layers;
  const int32_t *d = net->dims;

  std::vector<float *> G(L + 1, nullptr);
  for (int l = 1; l <= L; ++l)
    G[l] = (Jb_out && Jb_out[l - 1]) ? Jb_out[l - 1] : at(workspace, p.G[l]);

  // The rows of the softmax Jacobian of a narrow network: last layer, softmax, seed rows and the
  // cotangent step through the last layer in one launch, one workgroup per example.
  if (head == PFG_HEAD_SOFTMAX && !seeds && L >= 2) {
    GemmArgs g{};
    g.A = at(workspace, p.act[L - 1]); g.lda = d[L - 1]; g.a_batch_stride = d[L - 1]; g.S = 1; g.a_is_f32 = 1;
    g.W = net->W[L - 1]; g.ldw = d[L]; g.w_kn = 1; g.bf16 = (net->dtype == PFG_BF16);
    g.M = (int32_t)B; g.N = d[L]; g.K = d[L - 1];
    g.bias = bias_of(net, L); g.epilogue = EPI_HEAD;
    g.C2 = G[L]; g.ldc = d[L];
    const bool lower = lowest_requested(net, JW_out, Jb_out) < L;
    g.head_gprev = lower ? G[L - 1] : nullptr;
    g.head_mask = at(workspace, p.dphi[L - 1]);
    if (head_rows_applies(g)) {
      if ((rc = forward(net, X, B, L - 1, workspace, p, true, stream))) return rc;
      PFG_LAUNCH("gemm_forward", launch_head_rows(g, 1, stream));
      return weight_sweep(net, X, B, S, JW_out, Jb_out, G, workspace, p, stream, lower);
    }
  }

  if ((rc = forward(net, X, B, L, workspace, p, true, stream))) return rc;
  PFG_LAUNCH("seed_rows", launch_seed_rows(at(workspace, p.logits), seeds, seed_batch_stride, B, S,
                                           d[L], head, G[L], stream));
  return weight_sweep(net, X, B, S, JW_out, Jb_out, G, workspace, p, stream);
}

}  // extern "C"
