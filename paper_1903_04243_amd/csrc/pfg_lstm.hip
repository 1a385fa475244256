// C ABI of the unrolled LSTM: argument checks, workspace layout and the order in which the kernels
// are enqueued.  No arithmetic of the method happens on the host.
#include <algorithm>
#include <numeric>
#include <vector>

#include "../../include/pfg.h"
#include "common.h"
#include "host.h"

namespace {

using namespace pfg;

int check_lstm(const pfg_lstm *net) {
  if (!net) return fail(PFG_ERR_NULL, "net is NULL");
  if (net->input_size < 1 || net->state_size < 1 || net->output_size < 1 || net->steps < 1)
    return fail(PFG_ERR_SHAPE, "input_size %d, state_size %d, output_size %d and steps %d must all be >= 1",
                net->input_size, net->state_size, net->output_size, net->steps);
  constexpr int64_t kMaxDim = 1 << 22;
  if (net->input_size > kMaxDim || net->state_size > kMaxDim || net->output_size > kMaxDim ||
      net->steps > (1 << 16))
    return fail(PFG_ERR_SHAPE, "a size of the LSTM is out of range");
  if (net->dtype != PFG_F32)
    return fail(PFG_ERR_UNSUPPORTED, "the LSTM path is float32 only (dtype %d given)", net->dtype);
  if (!net->W) return fail(PFG_ERR_NULL, "net->W is NULL");
  if (!net->W_out) return fail(PFG_ERR_NULL, "net->W_out is NULL");
  return PFG_OK;
}

int check_lstm_rows(const pfg_lstm *net, int64_t B, int64_t S, bool grads) {
  if (B < 1) return fail(PFG_ERR_SHAPE, "B = %lld must be at least 1", (long long)B);
  if (S < 1) return fail(PFG_ERR_SHAPE, "S = %lld must be at least 1", (long long)S);
  const int64_t H = net->state_size, dx = net->input_size, T = net->steps, dy = net->output_size;
  if (B > kMaxRows || S > kMaxRows || B * S > kMaxRows || B * T > kMaxRows)
    return fail(PFG_ERR_OVERFLOW, "B * S = %lld * %lld or B * steps exceeds %lld rows", (long long)B,
                (long long)S, (long long)kMaxRows);
  const int64_t rows = B * S;
  if (4 * H > kMaxElems / (rows * (grads ? T : 1)) || T * dx > kMaxElems / rows ||
      rows * H > ((int64_t)1 << 38) || (dx + H) * 4 * H > 0x7fffffffLL || H * dy > 0x7fffffffLL ||
      (grads && (dx + H) * 4 * H > kMaxElems / B))
    return fail(PFG_ERR_OVERFLOW, "the tensors of this call exceed the indexing limits");
  return PFG_OK;
}

int check_lstm_seeds(const pfg_lstm *net, const float *seeds, int64_t S, int64_t stride) {
  const int64_t dy = net->output_size;
  if (!seeds) {
    if (S != dy)
      return fail(PFG_ERR_SHAPE, "identity seeds (seeds == NULL) need S == output_size, got S = %lld, output_size = %lld",
                  (long long)S, (long long)dy);
    return PFG_OK;
  }
  if (stride != 0 && stride < S * dy)
    return fail(PFG_ERR_SHAPE, "seed_batch_stride = %lld must be 0 or at least S * output_size = %lld",
                (long long)stride, (long long)(S * dy));
  return PFG_OK;
}

struct LstmPlan {
  size_t total = 0;
  size_t zx = 0, zh = 0, gates = 0, cs = 0, hs = 0;   // forward
  size_t y = 0, dy = 0, dh = 0, dc = 0, dz = 0, dz2 = 0, P = 0;
  size_t take(size_t bytes) {
    const size_t at = total;
    total += (bytes + 255) / 256 * 256;
    return at;
  }
};

LstmPlan make_lstm_plan(const pfg_lstm *net, int op, int64_t B, int64_t S) {
  const size_t H = net->state_size, T = net->steps, dy = net->output_size, f = sizeof(float);
  LstmPlan p;
  p.zx = p.take(f * B * T * 4 * H);
  p.zh = p.take(f * B * 4 * H);
  p.gates = p.take(f * B * T * 4 * H);
  p.cs = p.take(f * B * T * H);
  p.hs = p.take(f * B * T * H);
  if (op == PFG_LSTM_OP_PER_EXAMPLE_GRADS || op == PFG_LSTM_OP_GRAD_NORMS) {
    p.y = p.take(f * B * dy);
    p.dy = p.take(f * B * dy);
    p.dh = p.take(f * B * H);
    p.dc = p.take(f * B * H);
    p.dz = p.take(f * B * T * 4 * H);       // all steps are kept: the weight gradient sums over them
  } else {
    const size_t rows = (size_t)B * S;
    p.P = p.take(f * S * H);                // loop-invariant seeds pulled through the readout
    p.dh = p.take(f * rows * H);
    p.dc = p.take(f * rows * H);
    p.dz = p.take(f * rows * 4 * H);        // one step at a time, two buffers used alternately:
    p.dz2 = p.take(f * rows * 4 * H);       // a step's product reads one and fills the other
  }
  return p;
}

int check_ws(const LstmPlan &p, void *ws, size_t bytes) {
  if (!ws) return fail(PFG_ERR_WORKSPACE, "workspace is NULL (%zu bytes needed)", p.total);
  if (reinterpret_cast<uintptr_t>(ws) & 255)
    return fail(PFG_ERR_WORKSPACE, "workspace is not 256-byte aligned");
  if (bytes < p.total)
    return fail(PFG_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", bytes, p.total);
  return PFG_OK;
}

// Forward pass of all examples, all steps.  The input projections x_t W_x + b of every step do not
// depend on the recurrence and go out as ONE product over the B * T rows (Section 3.4: a matmul
// whose weight operand is loop-invariant folds the iteration index into its rows); only
// h_{t-1} W_h and the cell update remain on the sequential path.
int lstm_forward(const pfg_lstm *net, const void *X, int64_t B, void *ws, const LstmPlan &p,
                 hipStream_t stream) {
  const int32_t dx = net->input_size, H = net->state_size, T = net->steps;
  const float *W = static_cast<const float *>(net->W);
  {
    GemmArgs g{};
    g.A = X; g.lda = dx; g.a_batch_stride = dx; g.S = 1; g.a_is_f32 = 1;
    g.W = W; g.ldw = 4 * H; g.w_kn = 1;
    g.M = (int32_t)(B * T); g.N = 4 * H; g.K = dx;
    g.bias = net->b; g.epilogue = EPI_BIAS;
    g.C = ws_at(ws, p.zx); g.ldc = 4 * H;
    PFG_LAUNCH("lstm_gemm_input", launch_gemm(g, stream));
  }
  float *hs = ws_at(ws, p.hs);
  // With few rows every kernel on this sequential path is bound by launch and memory latency, so
  // the cell update rides in the epilogue of the recurrent product: one launch per step instead of
  // two: the small-problem kernel up to about 1000 rows (measured with a state of 256), the
  // LDS-tiled kernel with the same epilogue beyond.  Only a large batch whose state size is not a
  // multiple of 4 takes the LDS-tiled product and a separate cell kernel.
  const bool few_rows = (int64_t)((B + 63) / 64) * ((4 * (int64_t)H + 63) / 64) < 256;
  for (int t = 0; t < T; ++t) {
    if (t > 0) {
      GemmArgs g{};
      g.A = hs + (int64_t)(t - 1) * H; g.lda = (int64_t)T * H; g.a_batch_stride = (int64_t)T * H;
      g.S = 1; g.a_is_f32 = 1;
      g.W = W + (int64_t)dx * 4 * H; g.ldw = 4 * H; g.w_kn = 1;
      g.M = (int32_t)B; g.N = 4 * H; g.K = H;
      g.epilogue = EPI_LSTM_FWD;
      g.lstm_H = H; g.lstm_T = T; g.lstm_step = t;
      g.lstm_zx = ws_at(ws, p.zx); g.lstm_gates_w = ws_at(ws, p.gates);
      g.lstm_cs_w = ws_at(ws, p.cs); g.lstm_hs_w = hs;
      g.lstm_state_ld = (int64_t)T * H; g.lstm_state_ts = H; g.lstm_has_prev = 1;
      // fused on few rows (small-problem kernel) and on many when the tiled kernel takes the step
      if (few_rows || lstm_step_tiled_applies(g)) {
        PFG_LAUNCH("lstm_step", launch_gemm(g, stream));
        continue;
      }
    }
    if (t > 0) {
      GemmArgs g{};
      g.A = hs + (int64_t)(t - 1) * H; g.lda = (int64_t)T * H; g.a_batch_stride = (int64_t)T * H;
      g.S = 1; g.a_is_f32 = 1;
      g.W = W + (int64_t)dx * 4 * H; g.ldw = 4 * H; g.w_kn = 1;
      g.M = (int32_t)B; g.N = 4 * H; g.K = H;
      g.epilogue = EPI_NONE;
      g.C = ws_at(ws, p.zh); g.ldc = 4 * H;
      PFG_LAUNCH("lstm_gemm_recurrent", launch_gemm(g, stream));
    }
    PFG_LAUNCH("lstm_cell", launch_lstm_cell_forward(ws_at(ws, p.zx), t > 0 ? ws_at(ws, p.zh) : nullptr,
                                                     ws_at(ws, p.gates), ws_at(ws, p.cs), hs, B, H, T,
                                                     t, stream));
  }
  return PFG_OK;
}

// One reverse step as a single product.  With dz_t on `rows` rows (row m at dz + m * ld_dz):
//   [dx_t | dh_{t-1}] = dz_t [W_x ; W_h]^T
// The dx_t columns (only if J is given) go straight to their slot of the output; the dh_{t-1}
// columns are not stored: the epilogue carries each of them through the reverse cell update of
// step t - 1 and writes dz_{t-1} (row m at dz_prev + m * ld_dz_prev) and the running dc.
int reverse_step(const pfg_lstm *net, int t, const float *dz, int64_t ld_dz, int64_t rows, int64_t S,
                 float *J, float *dz_prev, int64_t ld_dz_prev, float *dc, void *ws, const LstmPlan &p,
                 hipStream_t stream) {
  const int32_t dx = net->input_size, H = net->state_size, T = net->steps;
  const float *W = static_cast<const float *>(net->W);
  GemmArgs g{};
  g.A = dz; g.lda = ld_dz; g.a_batch_stride = S * ld_dz; g.S = (int32_t)S; g.a_is_f32 = 1;
  g.ldw = 4 * H; g.w_kn = 0;
  g.M = (int32_t)rows; g.K = 4 * H;
  if (J) {
    g.C = J + (int64_t)t * dx; g.ldc = (int64_t)T * dx; g.streaming = 1;
  }
  if (t == 0) {                       // nothing precedes the first step: only dx_1 is wanted
    g.W = W; g.N = dx; g.epilogue = EPI_NONE;
    PFG_LAUNCH("lstm_gemm_reverse", launch_gemm(g, stream));
    return PFG_OK;
  }
  g.W = J ? W : W + (int64_t)dx * 4 * H;
  g.n_split = J ? dx : 0;
  g.N = g.n_split + H;
  g.epilogue = EPI_LSTM_BWD;
  g.lstm_H = H; g.lstm_T = T; g.lstm_step = t - 1;
  g.lstm_gates = ws_at(ws, p.gates); g.lstm_cs = ws_at(ws, p.cs);
  g.lstm_dc = dc; g.lstm_dz = dz_prev; g.lstm_dz_ld = ld_dz_prev;
  PFG_LAUNCH("lstm_gemm_reverse", launch_gemm(g, stream));
  return PFG_OK;
}

struct VarlenPlan {
  size_t total = 0;
  size_t zx = 0, state = 0, hfin = 0, idx = 0;
  size_t take(size_t bytes) {
    const size_t at = total;
    total += (bytes + 255) / 256 * 256;
    return at;
  }
};

VarlenPlan make_varlen_plan(const pfg_lstm *net, int64_t B, int64_t tokens) {
  const size_t H = net->state_size, f = sizeof(float);
  VarlenPlan p;
  p.zx = p.take(f * tokens * 4 * H);
  p.state = p.take(f * 3 * B * H);          // h (two buffers used alternately) and c, zeroed together
  p.hfin = p.take(f * B * H);               // last states in the caller's order, if h_out is not given
  p.idx = p.take(sizeof(int32_t) * 3 * B);  // first token row, original index, length of sorted row j
  return p;
}

struct WhilePlan {
  size_t total = 0;
  size_t zx = 0, state = 0, score = 0, hfin = 0, list = 0, meta = 0, flags = 0, cnt = 0, steps = 0;
  size_t zeroed = 0;      // floats from `state` on that the call zeroes in front of the loop
  // gradients only: history by token row, cotangents, head
  size_t gates = 0, cs = 0, hs = 0, dz = 0, dzp = 0, dh = 0, dc = 0, y = 0, gy = 0;
  size_t take(size_t bytes) {
    const size_t at = total;
    total += (bytes + 255) / 256 * 256;
    return at;
  }
};

// lists: how many active lists are kept (2: this trip's and the next one's, used alternately;
// max_steps + 1 with gradients: the list of every trip stays for the reverse sweep)
WhilePlan make_while_plan(const pfg_lstm *net, int64_t B, int64_t tokens, int64_t lists = 2, bool grads = false) {
  const size_t H = net->state_size, f = sizeof(float), i = sizeof(int32_t);
  const size_t tok = tokens > 0 ? tokens : 1;
  WhilePlan p;
  p.zx = p.take(f * tok * 4 * H);
  p.state = p.take(f * 3 * B * H);          // h (two buffers used alternately) and c, zeroed together
  // pieces of the halting score, one per group of 8 hidden units (lists of few rows only; zeroed with the state)
  const size_t pieces = B <= kWhileOneLaunchRows ? (size_t)B * ((H + 7) / 8) : 0;
  p.score = p.take(f * pieces);
  p.zeroed = (p.score + f * pieces - p.state) / f;
  p.hfin = p.take(f * B * H);               // last states, if h_out is not given
  p.list = p.take(i * lists * B);
  p.meta = p.take(i * 2 * lists);           // their {length, 0} descriptors
  p.flags = p.take(i * B);
  p.cnt = p.take(i * while_count_entries(B));
  p.steps = p.take(i * B);                  // trip counts, if steps_out is not given
  if (grads) {
    p.gates = p.take(f * tok * 4 * H);
    p.cs = p.take(f * tok * H);
    p.hs = p.take(f * tok * H);
    p.dz = p.take(f * tok * 4 * H);
    p.dh = p.take(f * B * H);               // cotangent of every iteration's final state
    p.dc = p.take(f * (B * H + 2 * B * 4 * H));   // dc, then dz by iteration (two buffers): zeroed together
    p.dzp = p.dc + f * B * H;
    p.y = p.take(f * B * net->output_size);
    p.gy = p.take(f * B * net->output_size);
  }
  return p;
}

int check_while_sizes(const pfg_lstm *net, int64_t B, int64_t tokens) {
  if (B < 1) return fail(PFG_ERR_SHAPE, "B = %lld must be at least 1", (long long)B);
  if (tokens < 0) return fail(PFG_ERR_SHAPE, "total_tokens = %lld is negative", (long long)tokens);
  const int64_t H = net->state_size;
  if (B > (1 << 24) || tokens > kMaxRows - (1 << 20) || (tokens > 0 && 4 * H > kMaxElems / tokens) ||
      B * H > ((int64_t)1 << 38))
    return fail(PFG_ERR_OVERFLOW, "B = %lld sequences with %lld tokens exceed the indexing limits",
                (long long)B, (long long)tokens);
  return PFG_OK;
}

// The part in front of the loop and the loop itself (Section 3.7), shared by the forward call and
// the gradient call.  With keep == false two lists are used alternately; with keep == true the list
// of every trip stays (list t + 1 holds the iterations that made trip t, meta t + 1 its length) and
// every trip also leaves its gate values, cell state and hidden state at the token row it consumed.
// On return trip t's hidden state of the rows that made it is in buffer t % 2 of p.state.
int while_forward_loop(const pfg_lstm *net, const void *X, const int32_t *seq_offsets, int64_t B,
                       int64_t total_tokens, int32_t max_steps, const float *halt_w, float halt_c, int32_t *steps,
                       int32_t *trips_out, void *ws, const WhilePlan &p, bool keep, hipStream_t stream) {
  const int32_t dx = net->input_size, H = net->state_size;
  const float *W = static_cast<const float *>(net->W);
  auto ints = [&](size_t off) { return reinterpret_cast<int32_t *>(static_cast<char *>(ws) + off); };

  // input projections of all tokens in one product (they do not depend on the recurrence), zero
  // states, the list of all iterations
  if (total_tokens > 0 && max_steps > 0) {
    GemmArgs g{};
    g.A = X; g.lda = dx; g.a_batch_stride = dx; g.S = 1; g.a_is_f32 = 1;
    g.W = W; g.ldw = 4 * H; g.w_kn = 1;
    g.M = (int32_t)total_tokens; g.N = 4 * H; g.K = dx;
    g.bias = net->b; g.epilogue = EPI_BIAS;
    g.C = ws_at(ws, p.zx); g.ldc = 4 * H;
    PFG_LAUNCH("lstm_gemm_input", launch_gemm(g, stream));
  }
  float *hbuf[2] = {ws_at(ws, p.state), ws_at(ws, p.state) + B * (int64_t)H};
  float *c = ws_at(ws, p.state) + 2 * B * (int64_t)H;
  PFG_LAUNCH("fill_zero", launch_fill_zero(ws_at(ws, p.state), (int64_t)p.zeroed, stream));
  // few rows and a condition on the state: the step kernel leaves the halting score of its new state in
  // pieces, and condition plus compaction of the next trip are one launch
  const bool pieces = halt_w && B <= kWhileOneLaunchRows;
  const int32_t nparts = (H + 7) / 8;
  auto list = [&](int32_t q) { return ints(p.list) + (keep ? q : (q & 1)) * B; };
  auto meta = [&](int32_t q) { return ints(p.meta) + 2 * (keep ? q : (q & 1)); };
  PFG_LAUNCH("while_select", launch_while_init(list(0), meta(0), steps, trips_out, (int32_t)B, max_steps, stream));

  // trip t evaluates the condition on the active rows, keeps those that go on, and runs the cell on
  // them; h_t goes to buffer t % 2 (a trip reads whole rows of h_{t-1} while other workgroups write
  // h_t), c is updated in place.  Every kernel takes the live row count from device memory; once the
  // list is empty the remaining trips find nothing to do.
  for (int32_t t = 0; t < max_steps; ++t) {
    PFG_LAUNCH("while_select",
               launch_while_select(list(t), meta(t), t, seq_offsets, (int32_t)total_tokens, hbuf[(t + 1) & 1], H,
                                   halt_w, halt_c, (int32_t)B, ints(p.flags), ints(p.cnt), list(t + 1), meta(t + 1),
                                   steps, trips_out, stream, pieces ? ws_at(ws, p.score) : nullptr, nparts));
    GemmArgs g{};
    g.A = hbuf[(t + 1) & 1]; g.lda = H; g.a_batch_stride = H; g.S = 1; g.a_is_f32 = 1;
    g.W = W + (int64_t)dx * 4 * H; g.ldw = 4 * H; g.w_kn = 1;
    g.M = (int32_t)B; g.N = 4 * H; g.K = H;
    g.epilogue = EPI_LSTM_FWD;
    g.lstm_H = H; g.lstm_T = 1; g.lstm_step = t;
    g.lstm_zx = ws_at(ws, p.zx); g.lstm_zx_rows = seq_offsets;
    g.lstm_gates_w = nullptr;
    g.lstm_cs_w = c; g.lstm_hs_w = hbuf[t & 1];
    g.lstm_state_ld = H; g.lstm_state_ts = 0; g.lstm_has_prev = 1;
    if (keep) {
      g.lstm_tok_gates = ws_at(ws, p.gates); g.lstm_tok_c = ws_at(ws, p.cs); g.lstm_tok_h = ws_at(ws, p.hs);
    }
    if (pieces) {
      g.lstm_halt_w = halt_w; g.lstm_score_part = ws_at(ws, p.score); g.lstm_score_ld = nparts;
    }
    g.sub = meta(t + 1); g.sub_rows = list(t + 1); g.sub_gather = 1; g.sub_scatter = 0; g.sub_offset_zero = 1;
    PFG_LAUNCH("lstm_step", launch_gemm(g, stream));
  }
  return PFG_OK;
}

// The gradient call keeps one list per trip and writes [B, dx + H, 4H] outputs one grid row per iteration.
int check_while_grads_sizes(const pfg_lstm *net, int64_t B, int64_t tokens, int32_t max_steps) {
  int rc = check_while_sizes(net, B, tokens);
  if (rc) return rc;
  if (max_steps < 0 || max_steps > (1 << 16))
    return fail(PFG_ERR_SHAPE, "max_steps = %d is outside [0, %d]", max_steps, 1 << 16);
  if (B > 65535) return fail(PFG_ERR_UNSUPPORTED, "gradients through the while loop take at most 65535 iterations (%lld given)", (long long)B);
  const int64_t H = net->state_size, dx = net->input_size;
  if ((dx + H) * 4 * H > kMaxElems / B || ((int64_t)max_steps + 1) * B > ((int64_t)1 << 31))
    return fail(PFG_ERR_OVERFLOW, "the tensors of this call exceed the indexing limits");
  return PFG_OK;
}

// Argument checks shared by the two calls that differentiate the while loop.
int check_while_grads_call(const pfg_lstm *net, const void *X, const int32_t *seq_offsets, const int32_t *labels,
                           int64_t B, int64_t total_tokens, int32_t max_steps) {
  int rc = check_lstm(net);
  if (rc) return rc;
  if (!X && total_tokens > 0) return fail(PFG_ERR_NULL, "X is NULL");
  if (!seq_offsets) return fail(PFG_ERR_NULL, "seq_offsets is NULL");
  if (!labels) return fail(PFG_ERR_NULL, "labels is NULL");
  return check_while_grads_sizes(net, B, total_tokens, max_steps);
}

int check_while_ws(const WhilePlan &p, const void *workspace, size_t workspace_bytes) {
  if (!workspace) return fail(PFG_ERR_WORKSPACE, "workspace is NULL (%zu bytes needed)", p.total);
  if (reinterpret_cast<uintptr_t>(workspace) & 255) return fail(PFG_ERR_WORKSPACE, "workspace is not 256-byte aligned");
  if (workspace_bytes < p.total)
    return fail(PFG_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, p.total);
  return PFG_OK;
}

// The loop, the head and -- if sweep -- the reverse loop of the gradient calls.  Leaves the last states
// in p.hfin, d ell / d y in gy, and with sweep the hidden states (p.hs) and dz (p.dz) of every trip by
// token row.
int while_sweeps(const pfg_lstm *net, const void *X, const int32_t *seq_offsets, const int32_t *labels, int64_t B,
                 int64_t total_tokens, int32_t max_steps, const float *halt_w, float halt_c, float *gy, float *loss_out,
                 int32_t *steps, bool sweep, void *ws, const WhilePlan &p, hipStream_t stream) {
  const int32_t dx = net->input_size, H = net->state_size, dy = net->output_size;
  auto ints = [&](size_t off) { return reinterpret_cast<int32_t *>(static_cast<char *>(ws) + off); };
  float *hbuf[2] = {ws_at(ws, p.state), ws_at(ws, p.state) + B * (int64_t)H};
  int rc = while_forward_loop(net, X, seq_offsets, B, total_tokens, max_steps, halt_w, halt_c, steps, nullptr, ws, p,
                              sweep, stream);
  if (rc) return rc;

  // ---- behind the loop: last states, readout, loss head ----
  float *hfin = ws_at(ws, p.hfin);
  PFG_LAUNCH("while_state", launch_while_state(steps, hbuf[0], hbuf[1], B, H, hfin, stream));
  {
    GemmArgs g{};
    g.A = hfin; g.lda = H; g.a_batch_stride = H; g.S = 1; g.a_is_f32 = 1;
    g.W = net->W_out; g.ldw = dy; g.w_kn = 1;
    g.M = (int32_t)B; g.N = dy; g.K = H;
    g.bias = net->b_out; g.ldc = dy;
    if (dy <= 32) {
      g.epilogue = EPI_HEAD; g.C = nullptr; g.C2 = gy; g.labels = labels; g.loss = loss_out;
      PFG_LAUNCH("lstm_gemm_readout", launch_gemm(g, stream));
    } else {
      g.epilogue = EPI_BIAS; g.C = ws_at(ws, p.y);
      PFG_LAUNCH("lstm_gemm_readout", launch_gemm(g, stream));
      PFG_LAUNCH("head", launch_head_softmax_ce(ws_at(ws, p.y), labels, B, dy, gy, loss_out, stream));
    }
  }
  if (!sweep) return PFG_OK;

  // ---- the reverse sweep.  Every iteration enters it at its own last trip with the cotangent of its
  // final state, dh = (d ell / d y) W_out^T, and dc = 0.  Reverse trip t runs on the list the forward
  // loop kept for trip t: one product carries dz_{t+1} W_h^T to the rows of that list (dz by iteration,
  // two buffers used alternately; the row of an iteration that made no trip t + 1 is still zero), and
  // its epilogue adds the seed where trip t is the iteration's last, updates dc and writes dz_t. ----
  float *seed = ws_at(ws, p.dh), *dc = ws_at(ws, p.dc), *dz = ws_at(ws, p.dz);
  float *dzi[2] = {ws_at(ws, p.dzp), ws_at(ws, p.dzp) + B * (int64_t)4 * H};
  {
    GemmArgs g{};
    g.A = gy; g.lda = dy; g.a_batch_stride = dy; g.S = 1; g.a_is_f32 = 1;
    g.W = net->W_out; g.ldw = dy; g.w_kn = 0;
    g.M = (int32_t)B; g.N = H; g.K = dy;
    g.epilogue = EPI_NONE; g.C = seed; g.ldc = H;
    PFG_LAUNCH("lstm_gemm_cotangent", launch_gemm(g, stream));
  }
  PFG_LAUNCH("fill_zero", launch_fill_zero(dc, B * (int64_t)H * 9, stream));
  const float *Wh = static_cast<const float *>(net->W) + (int64_t)dx * 4 * H;
  for (int32_t t = max_steps - 1; t >= 0; --t) {
    GemmArgs g{};
    g.A = dzi[(t + 1) & 1]; g.lda = 4 * H; g.a_batch_stride = 4 * H; g.S = 1; g.a_is_f32 = 1;
    g.W = Wh; g.ldw = 4 * H; g.w_kn = 0;
    g.M = (int32_t)B; g.N = H; g.K = 4 * H;
    g.epilogue = EPI_LSTM_BWD; g.n_split = 0;
    g.lstm_H = H; g.lstm_T = 1; g.lstm_step = t;
    g.lstm_gates = ws_at(ws, p.gates); g.lstm_cs = ws_at(ws, p.cs); g.lstm_zx_rows = seq_offsets;
    g.lstm_dc = dc; g.lstm_dz = dzi[t & 1]; g.lstm_dz_ld = 4 * H; g.lstm_tok_dz = dz;
    g.lstm_seed = seed; g.lstm_steps = steps;
    g.sub = ints(p.meta) + 2 * (t + 1); g.sub_rows = ints(p.list) + (int64_t)(t + 1) * B;
    g.sub_gather = 1; g.sub_scatter = 0; g.sub_rows_fastest = 1;
    PFG_LAUNCH("lstm_gemm_reverse", launch_gemm(g, stream));
  }
  return PFG_OK;
}

int check_varlen_sizes(const pfg_lstm *net, int64_t B, int64_t tokens) {
  if (B < 1) return fail(PFG_ERR_SHAPE, "B = %lld must be at least 1", (long long)B);
  if (tokens < B) return fail(PFG_ERR_SHAPE, "total_tokens = %lld is less than B = %lld", (long long)tokens, (long long)B);
  const int64_t H = net->state_size;
  if (B > kMaxRows || tokens > kMaxRows || 4 * H > kMaxElems / tokens || B * H > ((int64_t)1 << 38))
    return fail(PFG_ERR_OVERFLOW, "B = %lld sequences with %lld tokens exceed the indexing limits",
                (long long)B, (long long)tokens);
  return PFG_OK;
}

}  // namespace

extern "C" {

int pfg_lstm_varlen_workspace_bytes(const pfg_lstm *net, int64_t B, int64_t total_tokens, size_t *bytes) {
  clear_error();
  int rc = check_lstm(net);
  if (rc) return rc;
  if (!bytes) return fail(PFG_ERR_NULL, "bytes is NULL");
  if ((rc = check_varlen_sizes(net, B, total_tokens))) return rc;
  *bytes = make_varlen_plan(net, B, total_tokens).total;
  return PFG_OK;
}

int pfg_lstm_varlen_forward(const pfg_lstm *net, const void *X, const int32_t *lengths, int64_t B,
                            int64_t total_tokens, float *h_out, float *y_out, void *workspace,
                            size_t workspace_bytes, void *hip_stream) {
  clear_error();
  int rc = check_lstm(net);
  if (rc) return rc;
  if (!X) return fail(PFG_ERR_NULL, "X is NULL");
  if (!lengths) return fail(PFG_ERR_NULL, "lengths is NULL");
  if (!h_out && !y_out) return fail(PFG_ERR_NULL, "h_out and y_out are both NULL");
  if ((rc = check_varlen_sizes(net, B, total_tokens))) return rc;
  int64_t sum = 0;
  int32_t longest = 0;
  for (int64_t b = 0; b < B; ++b) {
    if (lengths[b] < 1) return fail(PFG_ERR_SHAPE, "lengths[%lld] = %d must be at least 1", (long long)b, lengths[b]);
    sum += lengths[b];
    longest = std::max(longest, lengths[b]);
  }
  if (sum != total_tokens)
    return fail(PFG_ERR_SHAPE, "the lengths add up to %lld, total_tokens is %lld", (long long)sum, (long long)total_tokens);
  const VarlenPlan p = make_varlen_plan(net, B, total_tokens);
  if (!workspace) return fail(PFG_ERR_WORKSPACE, "workspace is NULL (%zu bytes needed)", p.total);
  if (reinterpret_cast<uintptr_t>(workspace) & 255) return fail(PFG_ERR_WORKSPACE, "workspace is not 256-byte aligned");
  if (workspace_bytes < p.total)
    return fail(PFG_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, p.total);

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const int32_t dx = net->input_size, H = net->state_size, dy = net->output_size;
  const float *W = static_cast<const float *>(net->W);
  void *ws = workspace;

  // ---- active sets of all steps, from the lengths alone (host; index logic only) ----
  // order: sequences by decreasing length (ties by index); step t is active for the first
  // active[t] rows of that order.
  std::vector<int32_t> order(B);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return lengths[a] > lengths[b]; });
  std::vector<int64_t> first(B + 1, 0);
  for (int64_t b = 0; b < B; ++b) first[b + 1] = first[b] + lengths[b];
  // The staging array outlives the call: the asynchronous copy below may read it after the call
  // has returned.  An event recorded behind that copy guards the array: the next call on this
  // thread waits for it before it touches the array again (the copy is tiny, the wait all but
  // always over already).
  struct Staging {
    std::vector<int32_t> data;
    hipEvent_t copied = nullptr;
    bool pending = false;
  };
  thread_local Staging st;
  if (st.pending) {
    (void)hipEventSynchronize(st.copied);
    st.pending = false;
  }
  std::vector<int32_t> &staged = st.data;
  staged.resize(3 * B);
  for (int64_t j = 0; j < B; ++j) {
    staged[j] = (int32_t)first[order[j]];
    staged[B + j] = order[j];
    staged[2 * B + j] = lengths[order[j]];
  }
  std::vector<int64_t> active(longest);
  {
    int64_t n = B;
    for (int32_t t = 0; t < longest; ++t) {
      while (n > 0 && staged[2 * B + n - 1] <= t) --n;
      active[t] = n;
    }
  }
  int32_t *idx = reinterpret_cast<int32_t *>(static_cast<char *>(ws) + p.idx);
  hipError_t e = hipMemcpyAsync(idx, staged.data(), sizeof(int32_t) * 3 * B, hipMemcpyHostToDevice, stream);
  if (e != hipSuccess) return fail(PFG_ERR_DEVICE, "index upload: %s", hipGetErrorString(e));
  if (!st.copied && hipEventCreateWithFlags(&st.copied, hipEventDisableTiming) != hipSuccess) st.copied = nullptr;
  if (st.copied && hipEventRecord(st.copied, stream) == hipSuccess) {
    st.pending = true;
  } else if ((e = hipStreamSynchronize(stream)) != hipSuccess) {   // no event: wait for the copy here
    return fail(PFG_ERR_DEVICE, "index upload: %s", hipGetErrorString(e));
  }
  const int32_t *tok_row = idx, *orig = idx + B, *len_sorted = idx + 2 * B;

  // ---- input projections of all tokens in one product (no padding: M = total_tokens) ----
  {
    GemmArgs g{};
    g.A = X; g.lda = dx; g.a_batch_stride = dx; g.S = 1; g.a_is_f32 = 1;
    g.W = W; g.ldw = 4 * H; g.w_kn = 1;
    g.M = (int32_t)total_tokens; g.N = 4 * H; g.K = dx;
    g.bias = net->b; g.epilogue = EPI_BIAS;
    g.C = ws_at(ws, p.zx); g.ldc = 4 * H;
    PFG_LAUNCH("lstm_gemm_input", launch_gemm(g, stream));
  }
  float *hbuf[2] = {ws_at(ws, p.state), ws_at(ws, p.state) + B * (int64_t)H};
  float *c = ws_at(ws, p.state) + 2 * B * (int64_t)H;
  PFG_LAUNCH("fill_zero", launch_fill_zero(ws_at(ws, p.state), 3 * B * (int64_t)H, stream));

  // ---- the while loop: step t runs on the active prefix only; h_t goes to buffer t % 2 ----
  for (int32_t t = 0; t < longest; ++t) {
    GemmArgs g{};
    g.A = hbuf[(t + 1) & 1]; g.lda = H; g.a_batch_stride = H; g.S = 1; g.a_is_f32 = 1;
    g.W = W + (int64_t)dx * 4 * H; g.ldw = 4 * H; g.w_kn = 1;
    g.M = (int32_t)active[t]; g.N = 4 * H; g.K = H;
    g.epilogue = EPI_LSTM_FWD;
    g.lstm_H = H; g.lstm_T = 1; g.lstm_step = t;
    g.lstm_zx = ws_at(ws, p.zx); g.lstm_zx_rows = tok_row;
    g.lstm_gates_w = nullptr;
    g.lstm_cs_w = c; g.lstm_hs_w = hbuf[t & 1];
    g.lstm_state_ld = H; g.lstm_state_ts = 0; g.lstm_has_prev = 1;
    PFG_LAUNCH("lstm_step", launch_gemm(g, stream));
  }

  // ---- back to the caller's order: row j's last state sits in buffer (length - 1) % 2 ----
  // (parity[j] = length of sorted row j; odd lengths end in buffer 0)
  float *hfin = h_out ? h_out : ws_at(ws, p.hfin);
  PFG_LAUNCH("scatter_rows", launch_scatter_rows(hbuf[1], hbuf[0], len_sorted, orig, B, H, hfin, stream));
  if (y_out) {
    GemmArgs g{};
    g.A = hfin; g.lda = H; g.a_batch_stride = H; g.S = 1; g.a_is_f32 = 1;
    g.W = net->W_out; g.ldw = dy; g.w_kn = 1;
    g.M = (int32_t)B; g.N = dy; g.K = H;
    g.bias = net->b_out; g.epilogue = EPI_BIAS;
    g.C = y_out; g.ldc = dy;
    PFG_LAUNCH("lstm_gemm_readout", launch_gemm(g, stream));
  }
  return PFG_OK;
}

int pfg_lstm_while_workspace_bytes(const pfg_lstm *net, int64_t B, int64_t total_tokens, size_t *bytes) {
  clear_error();
  int rc = check_lstm(net);
  if (rc) return rc;
  if (!bytes) return fail(PFG_ERR_NULL, "bytes is NULL");
  if ((rc = check_while_sizes(net, B, total_tokens))) return rc;
  *bytes = make_while_plan(net, B, total_tokens).total;
  return PFG_OK;
}

int pfg_lstm_while_forward(const pfg_lstm *net, const void *X, const int32_t *seq_offsets, int64_t B,
                           int64_t total_tokens, int32_t max_steps, const float *halt_w, float halt_c,
                           float *h_out, float *y_out, int32_t *steps_out, int32_t *trips_out,
                           void *workspace, size_t workspace_bytes, void *hip_stream) {
  clear_error();
  int rc = check_lstm(net);
  if (rc) return rc;
  if (!X && total_tokens > 0) return fail(PFG_ERR_NULL, "X is NULL");
  if (!seq_offsets) return fail(PFG_ERR_NULL, "seq_offsets is NULL");
  if (!h_out && !y_out && !steps_out) return fail(PFG_ERR_NULL, "h_out, y_out and steps_out are all NULL");
  if (max_steps < 0 || max_steps > (1 << 20))
    return fail(PFG_ERR_SHAPE, "max_steps = %d is outside [0, %d]", max_steps, 1 << 20);
  if ((rc = check_while_sizes(net, B, total_tokens))) return rc;
  const WhilePlan p = make_while_plan(net, B, total_tokens);
  if (!workspace) return fail(PFG_ERR_WORKSPACE, "workspace is NULL (%zu bytes needed)", p.total);
  if (reinterpret_cast<uintptr_t>(workspace) & 255) return fail(PFG_ERR_WORKSPACE, "workspace is not 256-byte aligned");
  if (workspace_bytes < p.total)
    return fail(PFG_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, p.total);

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const int32_t H = net->state_size, dy = net->output_size;
  void *ws = workspace;
  auto ints = [&](size_t off) { return reinterpret_cast<int32_t *>(static_cast<char *>(ws) + off); };
  float *hbuf[2] = {ws_at(ws, p.state), ws_at(ws, p.state) + B * (int64_t)H};
  int32_t *steps = steps_out ? steps_out : ints(p.steps);
  if ((rc = while_forward_loop(net, X, seq_offsets, B, total_tokens, max_steps, halt_w, halt_c, steps, trips_out, ws, p,
                               false, stream)))
    return rc;

  // ---- behind the loop: every iteration's last state, then the readout on all rows ----
  float *hfin = h_out ? h_out : ws_at(ws, p.hfin);
  if (h_out || y_out)
    PFG_LAUNCH("while_state", launch_while_state(steps, hbuf[0], hbuf[1], B, H, hfin, stream));
  if (y_out) {
    GemmArgs g{};
    g.A = hfin; g.lda = H; g.a_batch_stride = H; g.S = 1; g.a_is_f32 = 1;
    g.W = net->W_out; g.ldw = dy; g.w_kn = 1;
    g.M = (int32_t)B; g.N = dy; g.K = H;
    g.bias = net->b_out; g.epilogue = EPI_BIAS;
    g.C = y_out; g.ldc = dy;
    PFG_LAUNCH("lstm_gemm_readout", launch_gemm(g, stream));
  }
  return PFG_OK;
}

int pfg_lstm_while_grads_workspace_bytes(const pfg_lstm *net, int64_t B, int64_t total_tokens, int32_t max_steps,
                                         size_t *bytes) {
  clear_error();
  int rc = check_lstm(net);
  if (rc) return rc;
  if (!bytes) return fail(PFG_ERR_NULL, "bytes is NULL");
  if ((rc = check_while_grads_sizes(net, B, total_tokens, max_steps))) return rc;
  *bytes = make_while_plan(net, B, total_tokens, (int64_t)max_steps + 1, true).total;
  return PFG_OK;
}

int pfg_lstm_while_per_example_grads(const pfg_lstm *net, const void *X, const int32_t *seq_offsets,
                                     const int32_t *labels, int64_t B, int64_t total_tokens, int32_t max_steps,
                                     const float *halt_w, float halt_c, float *dW_out, float *db_out,
                                     float *dWout_out, float *dbout_out, float *loss_out, int32_t *steps_out,
                                     void *workspace, size_t workspace_bytes, void *hip_stream) {
  clear_error();
  int rc = check_while_grads_call(net, X, seq_offsets, labels, B, total_tokens, max_steps);
  if (rc) return rc;
  if (!dW_out && !db_out && !dWout_out && !dbout_out && !loss_out)
    return fail(PFG_ERR_NULL, "dW_out, db_out, dWout_out, dbout_out and loss_out are all NULL");
  const WhilePlan p = make_while_plan(net, B, total_tokens, (int64_t)max_steps + 1, true);
  if ((rc = check_while_ws(p, workspace, workspace_bytes))) return rc;

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const int32_t dx = net->input_size, H = net->state_size, dy = net->output_size;
  void *ws = workspace;
  int32_t *steps = steps_out ? steps_out : reinterpret_cast<int32_t *>(static_cast<char *>(ws) + p.steps);
  float *gy = dbout_out ? dbout_out : ws_at(ws, p.gy);      // d ell / d y lands in dbout when given
  const bool sweep = dW_out || db_out;      // the reverse trips are needed for the cell's parameters only
  if ((rc = while_sweeps(net, X, seq_offsets, labels, B, total_tokens, max_steps, halt_w, halt_c, gy, loss_out, steps,
                         sweep, ws, p, stream)))
    return rc;
  if (dWout_out) {
    OuterArgs o{};
    o.a = ws_at(ws, p.hfin); o.lda = H; o.a_bf16 = 0; o.g = gy; o.ldg = dy; o.out = dWout_out;
    o.M = B; o.S = 1; o.d_in = H; o.d_out = dy;
    PFG_LAUNCH("outer_product", launch_outer(&o, 1, stream));
  }
  if (!sweep) return PFG_OK;
  // ---- per iteration, the sums over its own trips (the same W acts in every trip) ----
  PFG_LAUNCH("outer_sum_ragged",
             launch_outer_sum_ragged(static_cast<const float *>(X), dx, ws_at(ws, p.hs), H, ws_at(ws, p.dz), seq_offsets,
                                     steps, (int32_t)total_tokens, B, dW_out, db_out, stream));
  return PFG_OK;
}

int pfg_lstm_while_per_example_grad_norms(const pfg_lstm *net, const void *X, const int32_t *seq_offsets,
                                          const int32_t *labels, int64_t B, int64_t total_tokens, int32_t max_steps,
                                          const float *halt_w, float halt_c, float *sq_out, float *norm_out,
                                          float *loss_out, int32_t *steps_out, void *workspace,
                                          size_t workspace_bytes, void *hip_stream) {
  clear_error();
  int rc = check_while_grads_call(net, X, seq_offsets, labels, B, total_tokens, max_steps);
  if (rc) return rc;
  if (!sq_out && !norm_out) return fail(PFG_ERR_NULL, "sq_out and norm_out are both NULL");
  if (max_steps > kWhileNormMaxTrips)
    return fail(PFG_ERR_UNSUPPORTED, "gradient norms through the while loop take at most %d trips (max_steps = %d)",
                kWhileNormMaxTrips, max_steps);
  const WhilePlan p = make_while_plan(net, B, total_tokens, (int64_t)max_steps + 1, true);
  if ((rc = check_while_ws(p, workspace, workspace_bytes))) return rc;

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  void *ws = workspace;
  int32_t *steps = steps_out ? steps_out : reinterpret_cast<int32_t *>(static_cast<char *>(ws) + p.steps);
  float *gy = ws_at(ws, p.gy);
  if ((rc = while_sweeps(net, X, seq_offsets, labels, B, total_tokens, max_steps, halt_w, halt_c, gy, loss_out, steps,
                         true, ws, p, stream)))
    return rc;
  PFG_LAUNCH("while_grad_sqnorms",
             launch_while_grad_sqnorms(static_cast<const float *>(X), net->input_size, ws_at(ws, p.hs), net->state_size,
                                       ws_at(ws, p.dz), seq_offsets, steps, (int32_t)total_tokens, ws_at(ws, p.hfin), gy,
                                       net->output_size, B, sq_out, norm_out, stream));
  return PFG_OK;
}

int pfg_lstm_workspace_bytes(const pfg_lstm *net, int op, int64_t B, int64_t S, size_t *bytes) {
  clear_error();
  int rc = check_lstm(net);
  if (rc) return rc;
  if (!bytes) return fail(PFG_ERR_NULL, "bytes is NULL");
  if (op != PFG_LSTM_OP_PER_EXAMPLE_GRADS && op != PFG_LSTM_OP_JACOBIAN_INPUT && op != PFG_LSTM_OP_GRAD_NORMS)
    return fail(PFG_ERR_UNSUPPORTED, "unknown LSTM op %d", op);
  const bool grads = (op != PFG_LSTM_OP_JACOBIAN_INPUT);
  if (grads) S = 1;
  if ((rc = check_lstm_rows(net, B, S, grads))) return rc;
  *bytes = make_lstm_plan(net, op, B, S).total;
  return PFG_OK;
}

}  // extern "C"

namespace {

// Forward pass, readout and loss head (d ell / d y into gy), and -- if with_steps -- the reverse
// sweep that leaves dz_t of every step in the workspace (row b of step t at dz + b * T * 4H + t * 4H).
int lstm_forward_and_reverse(const pfg_lstm *net, const void *X, const int32_t *labels, int64_t B, float *gy,
                             float *loss_out, bool with_steps, void *ws, const LstmPlan &p,
                             hipStream_t stream) {
  const int32_t H = net->state_size, T = net->steps, dy = net->output_size;
  int rc = lstm_forward(net, X, B, ws, p, stream);
  if (rc) return rc;
  const float *hT = ws_at(ws, p.hs) + (int64_t)(T - 1) * H;
  {
    GemmArgs g{};
    g.A = hT; g.lda = (int64_t)T * H; g.a_batch_stride = (int64_t)T * H; g.S = 1; g.a_is_f32 = 1;
    g.W = net->W_out; g.ldw = dy; g.w_kn = 1;
    g.M = (int32_t)B; g.N = dy; g.K = H;
    g.bias = net->b_out; g.ldc = dy;
    if (dy <= 32) {
      g.epilogue = EPI_HEAD; g.C = nullptr; g.C2 = gy; g.labels = labels; g.loss = loss_out;
      PFG_LAUNCH("lstm_gemm_readout", launch_gemm(g, stream));
    } else {
      g.epilogue = EPI_BIAS; g.C = ws_at(ws, p.y);
      PFG_LAUNCH("lstm_gemm_readout", launch_gemm(g, stream));
      PFG_LAUNCH("head", launch_head_softmax_ce(ws_at(ws, p.y), labels, B, dy, gy, loss_out, stream));
    }
  }
  if (!with_steps) return PFG_OK;

  // dh_T = (d ell / d y) W_out^T, then back through the steps; dz of every step is kept
  float *dh = ws_at(ws, p.dh), *dc = ws_at(ws, p.dc), *dz = ws_at(ws, p.dz);
  {
    GemmArgs g{};
    g.A = gy; g.lda = dy; g.a_batch_stride = dy; g.S = 1; g.a_is_f32 = 1;
    g.W = net->W_out; g.ldw = dy; g.w_kn = 0;
    g.M = (int32_t)B; g.N = H; g.K = dy;
    g.epilogue = EPI_NONE; g.C = dh; g.ldc = H;
    PFG_LAUNCH("lstm_gemm_cotangent", launch_gemm(g, stream));
  }
  const int64_t ld_dz = (int64_t)T * 4 * H;
  PFG_LAUNCH("lstm_cell_backward",
             launch_lstm_cell_backward(dh, H, dc, 1, ws_at(ws, p.gates), ws_at(ws, p.cs), B, 1, H, T,
                                       T - 1, dz + (int64_t)(T - 1) * 4 * H, ld_dz, stream));
  for (int t = T - 1; t >= 1; --t)
    if ((rc = reverse_step(net, t, dz + (int64_t)t * 4 * H, ld_dz, B, 1, nullptr,
                           dz + (int64_t)(t - 1) * 4 * H, ld_dz, dc, ws, p, stream)))
      return rc;
  return PFG_OK;
}

}  // namespace

extern "C" {

int pfg_lstm_per_example_grads(const pfg_lstm *net, const void *X, const int32_t *labels, int64_t B,
                               float *dW_out, float *db_out, float *dWout_out, float *dbout_out,
                               float *loss_out, void *workspace, size_t workspace_bytes,
                               void *hip_stream) {
  clear_error();
  int rc = check_lstm(net);
  if (rc) return rc;
  if (!X) return fail(PFG_ERR_NULL, "X is NULL");
  if (!labels) return fail(PFG_ERR_NULL, "labels is NULL");
  if ((rc = check_lstm_rows(net, B, 1, true))) return rc;
  const LstmPlan p = make_lstm_plan(net, PFG_LSTM_OP_PER_EXAMPLE_GRADS, B, 1);
  if ((rc = check_ws(p, workspace, workspace_bytes))) return rc;

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const int32_t dx = net->input_size, H = net->state_size, T = net->steps, dy = net->output_size;
  void *ws = workspace;
  // d ell / d y lands in the caller's dbout when given
  float *gy = dbout_out ? dbout_out : ws_at(ws, p.dy);
  if ((rc = lstm_forward_and_reverse(net, X, labels, B, gy, loss_out, dW_out || db_out, ws, p, stream)))
    return rc;
  const float *hT = ws_at(ws, p.hs) + (int64_t)(T - 1) * H;
  if (dWout_out) {
    OuterArgs o{};
    o.a = hT; o.lda = (int64_t)T * H; o.a_bf16 = 0; o.g = gy; o.ldg = dy; o.out = dWout_out;
    o.M = B; o.S = 1; o.d_in = H; o.d_out = dy;
    PFG_LAUNCH("outer_product", launch_outer(&o, 1, stream));
  }
  if (!dW_out && !db_out) return PFG_OK;
  float *dz = ws_at(ws, p.dz);
  const int64_t ld_dz = (int64_t)T * 4 * H;
  if (dW_out) {
    // Both operands are stacked and the weights are shared by the steps: per example a product
    // with the step index as contraction.  Rows of x: all T steps of x_t^T dz_t.  Rows of h: steps
    // 2..T of h_{t-1}^T dz_t (h_0 = 0 contributes nothing).
    const int64_t out_bs = (int64_t)(dx + H) * 4 * H;
    OuterSumJob jobs[2] = {
        {static_cast<const float *>(X), (int64_t)T * dx, dx, dz, ld_dz, 4 * H, T, dx, dW_out},
        {ws_at(ws, p.hs), (int64_t)T * H, H, dz + 4 * H, ld_dz, 4 * H, T - 1, H,
         dW_out + (int64_t)dx * 4 * H}};
    PFG_LAUNCH("outer_sum", launch_outer_sum(jobs, 2, B, 4 * H, out_bs, stream));
  }
  if (db_out) PFG_LAUNCH("sum_steps", launch_sum_steps(dz, B, T, 4 * H, db_out, nullptr, stream));
  return PFG_OK;
}

int pfg_lstm_per_example_grad_norms(const pfg_lstm *net, const void *X, const int32_t *labels, int64_t B,
                                    float *sq_out, float *norm_out, float *loss_out, void *workspace,
                                    size_t workspace_bytes, void *hip_stream) {
  clear_error();
  int rc = check_lstm(net);
  if (rc) return rc;
  if (!X) return fail(PFG_ERR_NULL, "X is NULL");
  if (!labels) return fail(PFG_ERR_NULL, "labels is NULL");
  if (!sq_out && !norm_out) return fail(PFG_ERR_NULL, "sq_out and norm_out are both NULL");
  if (net->steps > kLstmNormMaxSteps)
    return fail(PFG_ERR_UNSUPPORTED, "gradient norms take at most %d steps (%d given)", kLstmNormMaxSteps,
                net->steps);
  if ((rc = check_lstm_rows(net, B, 1, true))) return rc;
  const LstmPlan p = make_lstm_plan(net, PFG_LSTM_OP_GRAD_NORMS, B, 1);
  if ((rc = check_ws(p, workspace, workspace_bytes))) return rc;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  void *ws = workspace;
  float *gy = ws_at(ws, p.dy);
  if ((rc = lstm_forward_and_reverse(net, X, labels, B, gy, loss_out, true, ws, p, stream))) return rc;
  PFG_LAUNCH("lstm_grad_sqnorms",
             launch_lstm_grad_sqnorms(static_cast<const float *>(X), ws_at(ws, p.hs), ws_at(ws, p.dz), gy, B,
                                      net->steps, net->input_size, net->state_size, net->output_size, sq_out,
                                      norm_out, stream));
  return PFG_OK;
}

int pfg_lstm_jacobian_input(const pfg_lstm *net, const void *X, int64_t B, const float *seeds,
                            int64_t S, int64_t seed_batch_stride, float *J_out, void *workspace,
                            size_t workspace_bytes, void *hip_stream) {
  clear_error();
  int rc = check_lstm(net);
  if (rc) return rc;
  if (!X) return fail(PFG_ERR_NULL, "X is NULL");
  if (!J_out) return fail(PFG_ERR_NULL, "J_out is NULL");
  if ((rc = check_lstm_rows(net, B, S, false))) return rc;
  if ((rc = check_lstm_seeds(net, seeds, S, seed_batch_stride))) return rc;
  const LstmPlan p = make_lstm_plan(net, PFG_LSTM_OP_JACOBIAN_INPUT, B, S);
  if ((rc = check_ws(p, workspace, workspace_bytes))) return rc;

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const int32_t dx = net->input_size, H = net->state_size, T = net->steps, dy = net->output_size;
  const int64_t rows = B * S;
  void *ws = workspace;
  if ((rc = lstm_forward(net, X, B, ws, p, stream))) return rc;

  // cotangent of the last state, dh_T[b, s, :] = seed row (b, s) W_out^T.  Loop-invariant seeds
  // (identity or shared) give one [S, H] block for all examples, which is not stacked: the first
  // reverse cell step reads it with batch stride 0.
  float *dh = ws_at(ws, p.dh), *dc = ws_at(ws, p.dc), *dz = ws_at(ws, p.dz);
  const float *dh_first;
  int64_t dh_first_bs;
  const bool shared = (seeds == nullptr) || (seed_batch_stride == 0);
  if (shared && !seeds) {
    PFG_LAUNCH("transpose", launch_transpose(net->W_out, 0, H, dy, ws_at(ws, p.P), stream));
    dh_first = ws_at(ws, p.P); dh_first_bs = 0;
  } else {
    GemmArgs g{};
    g.A = seeds; g.lda = dy; g.a_batch_stride = shared ? 0 : seed_batch_stride; g.S = (int32_t)S;
    g.a_is_f32 = 1;
    g.W = net->W_out; g.ldw = dy; g.w_kn = 0;
    g.M = (int32_t)(shared ? S : rows); g.N = H; g.K = dy;
    g.epilogue = EPI_NONE; g.C = shared ? ws_at(ws, p.P) : dh; g.ldc = H;
    PFG_LAUNCH("lstm_gemm_cotangent", launch_gemm(g, stream));
    dh_first = g.C; dh_first_bs = shared ? 0 : S * (int64_t)H;
  }

  float *dzs[2] = {dz, ws_at(ws, p.dz2)};
  int cur = 0;
  PFG_LAUNCH("lstm_cell_backward",
             launch_lstm_cell_backward(dh_first, dh_first_bs, dc, 1, ws_at(ws, p.gates),
                                       ws_at(ws, p.cs), rows, (int32_t)S, H, T, T - 1, dzs[cur], 4 * H,
                                       stream));
  for (int t = T - 1; t >= 0; --t) {
    if ((rc = reverse_step(net, t, dzs[cur], 4 * H, rows, S, J_out, dzs[cur ^ 1], 4 * H, dc, ws, p,
                           stream)))
      return rc;
    cur ^= 1;
  }
  return PFG_OK;
}

}  // extern "C"
