/*
 * pfg.h -- per-example gradients and Jacobians of a dense feed-forward network on one AMD
 * MI355X (gfx950), as a plain C ABI.
 *
 * What is computed is the result of the statically vectorised parallel-for of
 * "Auto-Vectorizing TensorFlow Graphs: Jacobians, Auto-Batching and Beyond" (arXiv 1903.04243)
 * for two of its uses: per-example gradients (Section 5.3) and Jacobians (Section 5.1).  The
 * result of pfor(body, n) is the body's output for iterations 0..n-1 stacked on a new leading
 * dimension (Section 4); every output below is laid out that way, iteration index first.
 *
 * Network.  L dense layers of widths d_0 -> d_1 -> ... -> d_L.
 *      a_0 = x,   z_l = a_{l-1} W_l + b_l,   a_l = phi(z_l) for l < L,   y = z_L
 *   W_l is row-major [d_{l-1}, d_l]; b_l is [d_l]; phi is one activation for all hidden layers.
 *
 * Memory.  Unless marked HOST, every pointer is a DEVICE pointer.  The caller owns every buffer
 * (inputs, outputs, workspace).  The library allocates no device memory, keeps no pointer after
 * a call returns, enqueues all work on the stream it is given and does not synchronise it.
 * Inputs are only read; requested outputs are overwritten in full (never accumulated into).
 * Outputs are always float32, row-major, last index fastest.  Buffers should be 16-byte aligned
 * (unaligned buffers are accepted and take a slower scalar path).
 *
 * Errors.  Every function returns a pfg_status.  All argument checks run on the host before
 * anything is enqueued, so a call that fails has not touched its outputs (PFG_ERR_DEVICE, a
 * failed kernel launch, is the one exception).  pfg_last_error() describes the last failure on
 * the calling thread.  No C++ exception crosses this boundary.  Label values are not checked
 * (they live on the device); a label outside [0, d_L) gives an unspecified gradient for that
 * example but no out-of-bounds access.
 */
#ifndef PFG_H_
#define PFG_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  PFG_OK = 0,
  PFG_ERR_NULL = -1,        /* a required pointer is NULL                                  */
  PFG_ERR_SHAPE = -2,       /* a size, stride or count is out of range or inconsistent     */
  PFG_ERR_UNSUPPORTED = -3, /* unknown activation, dtype, head or op                       */
  PFG_ERR_WORKSPACE = -4,   /* workspace NULL, misaligned (256 B) or too small             */
  PFG_ERR_OVERFLOW = -5,    /* a tensor would have more elements than the kernels index    */
  PFG_ERR_DEVICE = -6       /* the HIP runtime reported an error                           */
} pfg_status;

/* Hidden activation phi.  ReLU'(0) is taken as 0.  GELU is the exact form z * Phi(z) with the
 * normal CDF Phi, derivative Phi(z) + z * exp(-z^2 / 2) / sqrt(2 pi). */
typedef enum { PFG_ACT_IDENTITY = 0, PFG_ACT_RELU = 1, PFG_ACT_TANH = 2, PFG_ACT_GELU_ERF = 3 } pfg_act;

/* Element type of X, W_l and b_l.  With PFG_BF16 the matrix products run on bf16 operands
 * (hidden activations and cotangents are rounded to bf16 when they feed a product) with float32
 * accumulation; everything written out is the float32 accumulator value. */
typedef enum { PFG_F32 = 0, PFG_BF16 = 1 } pfg_dtype;

/* Which vector the seed rows of pfg_jacobian_weights are contracted with: the logits y, or
 * softmax(y). */
typedef enum { PFG_HEAD_LOGITS = 0, PFG_HEAD_SOFTMAX = 1 } pfg_head;

typedef enum {
  PFG_OP_PER_EXAMPLE_GRADS = 0,
  PFG_OP_JACOBIAN_INPUT = 1,
  PFG_OP_JACOBIAN_WEIGHTS = 2,
  PFG_OP_GRAD_NORMS = 3,
  PFG_OP_HESSIAN_INPUT = 4
} pfg_op;

typedef struct {
  int32_t num_layers;     /* L >= 1                                                         */
  const int32_t *dims;    /* HOST, L+1 entries d_0..d_L, each >= 1                          */
  const void *const *W;   /* HOST array of L device pointers; W[l-1] is W_l [d_{l-1}, d_l]  */
  const void *const *b;   /* HOST array of L device pointers or NULL; a NULL array or a NULL
                             entry means a zero bias                                        */
  int32_t hidden_act;     /* pfg_act, applied after layers 1..L-1, never after layer L      */
  int32_t dtype;          /* pfg_dtype of X, W_l, b_l                                       */
} pfg_mlp;

/* Bytes of workspace the given op needs for batch B and S seed rows per example (S is ignored
 * by PFG_OP_PER_EXAMPLE_GRADS and PFG_OP_GRAD_NORMS).  The figure covers the case where no optional output is given;
 * it is a multiple of 256 and never 0.  The workspace passed to an op must be 256-byte aligned. */
int pfg_workspace_bytes(const pfg_mlp *net, int op, int64_t B, int64_t S, size_t *bytes);

/* Per-example gradients (Section 5.3): iteration b of the parallel-for computes the gradient of
 * example b's own loss  ell_b = -log softmax(y_b)[labels[b]]  (not divided by B), so
 *      dW_out[l-1][b, i, j] = d ell_b / d W_l[i, j] = a_{l-1}[b, i] * delta_l[b, j]
 *      db_out[l-1][b, j]    = d ell_b / d b_l[j]    = delta_l[b, j]
 *      loss_out[b]          = ell_b
 * with delta_L = softmax(y_b) - onehot(labels[b]) and
 * delta_{l-1} = (delta_l W_l^T) * phi'(z_{l-1}).  Contributions of different examples are kept
 * separate; summing dW_out[l-1] over b gives the gradient of the summed loss.
 *   X       [B, d_0], element type net->dtype
 *   labels  [B] int32
 *   dW_out  HOST array of L device pointers, entry l-1 is [B, d_{l-1}, d_l]; a NULL array or
 *           entry skips that output
 *   db_out  HOST array of L device pointers, entry l-1 is [B, d_l]; NULL skips
 *   loss_out [B] or NULL */
int pfg_per_example_grads(const pfg_mlp *net, const void *X, const int32_t *labels, int64_t B,
                          float *const *dW_out, float *const *db_out, float *loss_out,
                          void *workspace, size_t workspace_bytes, void *hip_stream);

/* Input Jacobian (Section 5.1: a parallel-for in which every iteration is the gradient of one
 * scalar of the output), nested inside the parallel-for over examples (Section 3.7):
 *      J_out[b, s, i] = d <seed row s of example b, y_b> / d x_b[i]
 * Only the diagonal blocks (output of example b with respect to input of example b) exist; the
 * others are identically zero and are not produced.
 *   seeds   NULL: the identity, S must equal d_L, so J_out[b, s, i] = d y_b[s] / d x_b[i].
 *           Otherwise float32 rows of length d_L: example b reads rows
 *           seeds + b * seed_batch_stride + s * d_L.  seed_batch_stride == 0 shares one [S, d_L]
 *           block between all examples (a loop-invariant operand is not stacked, Section 3.4);
 *           otherwise it must be >= S * d_L.
 *   J_out   [B, S, d_0] */
int pfg_jacobian_input(const pfg_mlp *net, const void *X, int64_t B, const float *seeds,
                       int64_t S, int64_t seed_batch_stride, float *J_out, void *workspace,
                       size_t workspace_bytes, void *hip_stream);

/* Jacobian with respect to the weights (the same nesting, differentiating with respect to the
 * loop-invariant W_l and b_l; the per-iteration results stay separate):
 *      JW_out[l-1][b, s, i, j] = d <seed row s, h(y_b)> / d W_l[i, j] = a_{l-1}[b, i] * G_l[b, s, j]
 *      Jb_out[l-1][b, s, j]    = G_l[b, s, j]
 * where h is the identity (PFG_HEAD_LOGITS) or softmax (PFG_HEAD_SOFTMAX), G_L[b, s, :] is the
 * seed row pulled back through h, and G_{l-1} = (G_l W_l^T) * phi'(z_{l-1}).  With head =
 * SOFTMAX and seeds = NULL, row s is the gradient of softmax(y_b)[s].
 *   seeds, S, seed_batch_stride   as for pfg_jacobian_input
 *   JW_out  HOST array of L device pointers, entry l-1 is [B, S, d_{l-1}, d_l]; NULL skips
 *   Jb_out  HOST array of L device pointers, entry l-1 is [B, S, d_l]; NULL skips */
int pfg_jacobian_weights(const pfg_mlp *net, const void *X, int64_t B, int head,
                         const float *seeds, int64_t S, int64_t seed_batch_stride,
                         float *const *JW_out, float *const *Jb_out, void *workspace,
                         size_t workspace_bytes, void *hip_stream);

/* pfg_per_example_grads for callers that cannot allocate device memory or have no workspace to
 * hand over: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, kernels and results as pfg_per_example_grads, without the workspace: the
 * intermediate tensors live in a buffer of PFG_STATIC_SCRATCH_BYTES that is part of the library's
 * device image (one copy per GPU, resident from the time the library is loaded on that GPU until
 * the process ends).  The call allocates and frees no device memory.
 *   - A network and batch that need more (pfg_workspace_bytes reports the figure) are rejected
 *     with PFG_ERR_WORKSPACE before anything is enqueued.
 *   - All calls on one GPU share that GPU's buffer: calls that overlap on one GPU (two streams, two
 *     threads) race; calls on one stream are ordered by the stream.  Nothing in the buffer has to
 *     be zero at entry and nothing is kept between calls.
 *   - The first call on a GPU looks up the buffer's address (no allocation, but a runtime query):
 *     make one call outside graph capture before capturing. */
#define PFG_STATIC_SCRATCH_BYTES (64u << 20)
int pfg_per_example_grads_static(const pfg_mlp *net, const void *X, const int32_t *labels, int64_t B,
                                 float *const *dW_out, float *const *db_out, float *loss_out,
                                 void *hip_stream);

/* Norms of the per-example gradients of Section 5.3 without writing the gradients out (the
 * statistic that per-example clipping and importance weighting need).  The gradient of layer l
 * for example b is the product of a column a_{l-1}[b, :] and a row delta_l[b, :] -- the matmul
 * with both operands stacked (Section 3.4) and contraction length 1 -- so its squared Frobenius
 * norm is |a_{l-1}[b]|^2 |delta_l[b]|^2 and never needs the [B, d_{l-1}, d_l] tensor:
 *      sq_layers_out[b, l-1] = sum_ij dW_l[b,i,j]^2 + (layer l has a bias ? sum_j db_l[b,j]^2 : 0)
 *      norm_out[b]           = sqrt(sum_l sq_layers_out[b, l-1])
 * A layer "has a bias" when net->b and net->b[l-1] are non-NULL.
 *   X, labels, loss_out   as for pfg_per_example_grads
 *   sq_layers_out [B, L] or NULL;  norm_out [B] or NULL (at least one of the two is required) */
int pfg_per_example_grad_norms(const pfg_mlp *net, const void *X, const int32_t *labels, int64_t B,
                               float *sq_layers_out, float *norm_out, float *loss_out,
                               void *workspace, size_t workspace_bytes, void *hip_stream);

/* Input Hessian as the Jacobian of the Jacobian (Section 5.1 names Hessians of non-scalar outputs
 * as a use of the nested parallel-for): every scalar of pfg_jacobian_input's result is
 * differentiated once more with respect to the example's own input,
 *      H_out[b, s, i, j] = d J[b, s, i] / d x_b[j] = d^2 <seed row s of example b, y_b> / d x_b[i] d x_b[j].
 * With T_l[b] = d z_l[b] / d x_b (a [d_l, d_0] matrix, T_1 = W_1^T, T_{l+1} = W_{l+1}^T diag(phi'(z_l)) T_l)
 * and h_l[b, s, :] the cotangent of the seed row at a_l, the result is
 *      H[b, s] = sum_{l < L} T_l[b]^T diag(h_l[b, s, :] * phi''(z_l[b, :])) T_l[b],
 * one batched matrix product per call (both operands depend on b).  It is identically zero for
 * PFG_ACT_IDENTITY and PFG_ACT_RELU (phi'' = 0, also at the kink) and for L = 1.
 *   net->dtype PFG_BF16: the three sweeps (forward, tangents, cotangents) run their products on bf16
 *   operands as the other calls do; the tangents, the curvature weights and the batched product that
 *   forms H stay float32
 *   seeds, S, seed_batch_stride   as for pfg_jacobian_input
 *   H_out   [B, S, d_0, d_0] */
int pfg_hessian_input(const pfg_mlp *net, const void *X, int64_t B, const float *seeds, int64_t S,
                      int64_t seed_batch_stride, float *H_out, void *workspace,
                      size_t workspace_bytes, void *hip_stream);

/* ------------------------------------------------------------------------------------------
 * Statically unrolled LSTM (the model of the paper's own per-example-gradient and Jacobian
 * benchmarks, Sections 6.1, 6.3 and 6.4: a single-layer unidirectional RNN, every example a
 * complete sequence, unrolled to a fixed number of steps).
 *      u_t = [x_t, h_{t-1}],   z_t = u_t W + b,   W row-major [input_size + state_size, 4 state_size]
 *      column blocks of W and b in the order i, g, f, o:
 *      i = sigmoid(z_i), g = tanh(z_g), f = sigmoid(z_f), o = sigmoid(z_o)
 *      c_t = f c_{t-1} + i g,   h_t = o tanh(c_t),   h_0 = c_0 = 0
 *      y = h_T W_out + b_out,   W_out row-major [state_size, output_size]
 * A sequence is one parallel-for iteration: X is [B, steps, input_size], example index first.
 * All tensors are float32 (dtype must be PFG_F32).
 * ---------------------------------------------------------------------------------------- */
typedef struct {
  int32_t input_size;   /* >= 1 */
  int32_t state_size;   /* >= 1 */
  int32_t output_size;  /* >= 1 */
  int32_t steps;        /* T >= 1 */
  const void *W;        /* DEVICE [input_size + state_size, 4 * state_size] */
  const void *b;        /* DEVICE [4 * state_size] or NULL (zero bias)      */
  const void *W_out;    /* DEVICE [state_size, output_size]                 */
  const void *b_out;    /* DEVICE [output_size] or NULL (zero bias)         */
  int32_t dtype;        /* PFG_F32                                          */
} pfg_lstm;

typedef enum {
  PFG_LSTM_OP_PER_EXAMPLE_GRADS = 0,
  PFG_LSTM_OP_JACOBIAN_INPUT = 1,
  PFG_LSTM_OP_GRAD_NORMS = 2
} pfg_lstm_op;

/* Workspace bytes of an LSTM op (S is ignored by PFG_LSTM_OP_PER_EXAMPLE_GRADS); a multiple of
 * 256, never 0. */
int pfg_lstm_workspace_bytes(const pfg_lstm *net, int op, int64_t B, int64_t S, size_t *bytes);

/* Per-example gradients (Section 5.3) of ell_b = -log softmax(y_b)[labels[b]] (not divided by B).
 * The same W acts at every step, so an example's gradient with respect to W is the sum over the
 * steps of that step's outer product (contributions of different examples stay separate):
 *      dW_out[b]     = sum_t u_t[b]^T dz_t[b]          [B, input_size + state_size, 4 state_size]
 *      db_out[b]     = sum_t dz_t[b]                   [B, 4 state_size]
 *      dWout_out[b]  = h_T[b]^T (softmax(y_b) - onehot)  [B, state_size, output_size]
 *      dbout_out[b]  = softmax(y_b) - onehot           [B, output_size]
 *      loss_out[b]   = ell_b
 * where dz_t is the cotangent of z_t from back-propagation through the unrolled steps.  Any output
 * pointer may be NULL (skipped). */
int pfg_lstm_per_example_grads(const pfg_lstm *net, const void *X, const int32_t *labels, int64_t B,
                               float *dW_out, float *db_out, float *dWout_out, float *dbout_out,
                               float *loss_out, void *workspace, size_t workspace_bytes,
                               void *hip_stream);

/* Norms of the per-example gradients above without writing the gradients out (as
 * pfg_per_example_grad_norms does for the dense network).  The weight gradient is a sum over the
 * steps of outer products, dW[b] = sum_t u_t[b]^T dz_t[b], so its squared Frobenius norm is
 *      |dW[b]|^2 = sum_{t, t'} (u_t[b] . u_t'[b]) (dz_t[b] . dz_t'[b])
 * -- two steps x steps Gram matrices per example instead of an [input_size + state_size,
 * 4 state_size] matrix --, and likewise |db[b]|^2 = sum_{t, t'} dz_t[b] . dz_t'[b].
 *      sq_out[b, 0..3] = |dW[b]|^2, |db[b]|^2, |dWout[b]|^2, |dbout[b]|^2
 *      norm_out[b]     = sqrt of their sum
 * steps is limited to 64.  sq_out [B, 4] or NULL; norm_out [B] or NULL (at least one of the two);
 * loss_out [B] or NULL. */
int pfg_lstm_per_example_grad_norms(const pfg_lstm *net, const void *X, const int32_t *labels, int64_t B,
                                    float *sq_out, float *norm_out, float *loss_out, void *workspace,
                                    size_t workspace_bytes, void *hip_stream);

/* Input Jacobian (Section 5.1 nested in the loop over examples, Section 3.7):
 *      J_out[b, s, t, i] = d <seed row s of example b, y_b> / d x_b[t, i]     [B, S, steps, input_size]
 * seeds, S, seed_batch_stride as for pfg_jacobian_input (rows of length output_size). */
int pfg_lstm_jacobian_input(const pfg_lstm *net, const void *X, int64_t B, const float *seeds,
                            int64_t S, int64_t seed_batch_stride, float *J_out, void *workspace,
                            size_t workspace_bytes, void *hip_stream);

/* Sequences of different lengths (the auto-batching LSTM workload of Section 6.2: every sequence
 * is iterated to its own length, inputs are not padded).  The body of the parallel-for holds a
 * sequential while loop, "while t < length_i: (h, c) = cell(x_i[t], h, c)"; its vectorised form
 * (Section 3.7) keeps the set of iterations that are still active and runs each step on those only.
 * The loop condition depends on the lengths and the step counter alone, so all active sets are
 * known before the loop starts: the sequences are ordered by decreasing length once, which makes
 * every active set a prefix of that order, and the results are put back in the caller's order at
 * the end.  net->steps is ignored.
 *   X               DEVICE [sum of lengths, input_size]: the tokens of sequence 0, then sequence 1, ...
 *   lengths         HOST   [B] int32, each >= 1 (read before the call returns)
 *   total_tokens    sum of lengths (checked)
 *   h_out           DEVICE [B, state_size] or NULL: hidden state of each sequence after its last token
 *   y_out           DEVICE [B, output_size] or NULL: h_out W_out + b_out
 * The call copies three small index arrays to the workspace with an asynchronous copy on the
 * stream (from a host buffer the library keeps per calling thread and guards with an event, so
 * calls may follow each other without synchronising); do not capture it into a graph.  For lengths
 * that live on the device, or a loop that also stops on a condition of the state, see
 * pfg_lstm_while_forward. */
int pfg_lstm_varlen_workspace_bytes(const pfg_lstm *net, int64_t B, int64_t total_tokens, size_t *bytes);
int pfg_lstm_varlen_forward(const pfg_lstm *net, const void *X, const int32_t *lengths, int64_t B,
                            int64_t total_tokens, float *h_out, float *y_out, void *workspace,
                            size_t workspace_bytes, void *hip_stream);

/* A while loop whose condition depends on the state, nested in the parallel-for, converted by the
 * rule of Section 3.7: the vectorised loop keeps the list I of the iterations that are still
 * active; every trip evaluates the condition on the rows of I only, keeps the rows for which it
 * holds, and runs the body on those.  Iteration i (one sequence) is
 *      h = c = 0, t = 0
 *      while t < length_i and t < max_steps and halt_c + sum_k h[k] * halt_w[k] <= 0:
 *          (h, c) = cell(x_i[t], h, c);  t = t + 1
 *      y_i = h W_out + b_out
 * The condition is evaluated before every trip, also the first (with h = 0); a score of exactly 0
 * lets the loop go on.  The list, its length and the trip counts live in device memory: the call
 * enqueues max_steps trips whose kernels read the live length themselves and do nothing once the
 * list is empty, copies nothing from or to the host and does not synchronise, so it can be captured
 * into a graph.  net->steps is ignored.
 *   X             DEVICE [total_tokens, input_size]: the tokens of all sequences
 *   seq_offsets   DEVICE [B + 1] int32: sequence i owns rows seq_offsets[i] .. seq_offsets[i + 1] - 1
 *                 of X (length 0 is allowed).  The values are not checked on the host; a range that
 *                 leaves [0, total_tokens] is cut to it, so no row outside X is ever read
 *   total_tokens  rows of X (HOST value, sizes the input projection)
 *   max_steps     HOST, >= 0: cap on the trips of every iteration, and the number of trips enqueued
 *   halt_w        DEVICE [state_size] float32, or NULL (the score is then halt_c alone)
 *   h_out         DEVICE [B, state_size] or NULL: the state each iteration left the loop with
 *   y_out         DEVICE [B, output_size] or NULL
 *   steps_out     DEVICE [B] int32 or NULL: trips made by each iteration
 *   trips_out     DEVICE [1] int32 or NULL: trips of the vectorised loop whose list was not empty
 * (at least one of h_out, y_out, steps_out is required).  The halting decision is taken in float32. */
int pfg_lstm_while_workspace_bytes(const pfg_lstm *net, int64_t B, int64_t total_tokens, size_t *bytes);
int pfg_lstm_while_forward(const pfg_lstm *net, const void *X, const int32_t *seq_offsets, int64_t B,
                           int64_t total_tokens, int32_t max_steps, const float *halt_w, float halt_c,
                           float *h_out, float *y_out, int32_t *steps_out, int32_t *trips_out,
                           void *workspace, size_t workspace_bytes, void *hip_stream);

/* Per-example gradients (Section 5.3) of a body that holds the while loop above (Section 3.7):
 * iteration i runs the loop of pfg_lstm_while_forward on its own tokens (T_i trips), then
 *      ell_i = -log softmax(h W_out + b_out)[labels[i]]
 * and the call returns the gradient of ell_i with respect to W, b, W_out, b_out for every i.  The
 * loop condition is a comparison and has no derivative: the gradient is that of the T_i cell
 * applications the iteration made, taken in reverse.  The vectorised reverse loop runs trip
 * t = max_steps - 1 .. 0 on the list of iterations the forward loop kept for that trip (an
 * iteration enters the reverse loop at its own last trip; until then its cotangent keeps the seed
 * (d ell / d y) W_out^T), and sums every iteration's outer products over its own trips only.
 * Arguments as for pfg_lstm_while_forward, and
 *   labels        DEVICE [B] int32 in [0, output_size)
 *   max_steps     HOST, 0 .. 65536
 *   dW_out        DEVICE [B, input_size + state_size, 4 * state_size] or NULL
 *   db_out        DEVICE [B, 4 * state_size] or NULL
 *   dWout_out     DEVICE [B, state_size, output_size] or NULL
 *   dbout_out     DEVICE [B, output_size] or NULL
 *   loss_out      DEVICE [B] or NULL
 *   steps_out     DEVICE [B] int32 or NULL: T_i
 * (at least one of the five float outputs is required; B <= 65535).  An iteration with T_i = 0 has
 * dW = db = dWout = 0 and dbout = softmax(b_out) - onehot.  Every output element is written.  The
 * workspace keeps one list per trip and the gate values, cell and hidden states by token row; like the
 * forward call this one copies nothing from or to the host and does not synchronise. */
int pfg_lstm_while_grads_workspace_bytes(const pfg_lstm *net, int64_t B, int64_t total_tokens, int32_t max_steps,
                                         size_t *bytes);
int pfg_lstm_while_per_example_grads(const pfg_lstm *net, const void *X, const int32_t *seq_offsets,
                                     const int32_t *labels, int64_t B, int64_t total_tokens, int32_t max_steps,
                                     const float *halt_w, float halt_c, float *dW_out, float *db_out,
                                     float *dWout_out, float *dbout_out, float *loss_out, int32_t *steps_out,
                                     void *workspace, size_t workspace_bytes, void *hip_stream);

/* Norms of those per-example gradients without the gradients (what per-example clipping needs,
 * Section 5.3): the same forward and reverse loops, then per iteration, with u_t = [x_t | h_{t-1}]
 * and dz_t the cotangent of the gate pre-activations of its trip t,
 *      |dW|^2 = |sum_t u_t^T dz_t|^2 = sum_{t, t'} (u_t . u_t') (dz_t . dz_t'),    |db|^2 = sum_{t, t'} dz_t . dz_t',
 *      |dWout|^2 = |h|^2 |d ell / d y|^2,    |dbout|^2 = |d ell / d y|^2
 * from two T_i x T_i Gram matrices per iteration; the stacked gradient [B, input_size + state_size,
 * 4 * state_size] is never written.  Arguments as for pfg_lstm_while_per_example_grads, and
 *   max_steps     HOST, 0 .. 128
 *   sq_out        DEVICE [B, 4] or NULL: |dW|^2, |db|^2, |dWout|^2, |dbout|^2
 *   norm_out      DEVICE [B] or NULL: the root of their sum           (at least one of the two)
 *   loss_out      DEVICE [B] or NULL;  steps_out  DEVICE [B] int32 or NULL
 * Workspace: pfg_lstm_while_grads_workspace_bytes. */
int pfg_lstm_while_per_example_grad_norms(const pfg_lstm *net, const void *X, const int32_t *seq_offsets,
                                          const int32_t *labels, int64_t B, int64_t total_tokens, int32_t max_steps,
                                          const float *halt_w, float halt_c, float *sq_out, float *norm_out,
                                          float *loss_out, int32_t *steps_out, void *workspace,
                                          size_t workspace_bytes, void *hip_stream);

/* ------------------------------------------------------------------------------------------
 * Convolutional network of the paper's MNIST benchmarks (Section 6.1: conv-relu-maxpool blocks
 * followed by dense layers; the dropout of that model is a stateful random op and is left out).
 * Images are [height, width, channels], channel index fastest.  Conv block i:
 *      z[y, x, co] = bc[co] + sum_{ky, kx, ci} in[y + ky - p, x + kx - p, ci] * Wc[ky, kx, ci, co]
 *      p = (k - 1) / 2, k odd, zero outside the image; a = relu(z); 2 x 2 max-pooling, stride 2
 *      (the height and width entering every block must be even)
 * The last block's output, flattened in (y, x, c) order, is the input of `dense`
 * (dense.dims[0] must equal its size; dense.dtype must be PFG_F32).
 * ---------------------------------------------------------------------------------------- */
typedef struct {
  int32_t height, width, channels;
  int32_t num_conv;          /* >= 1 */
  const int32_t *kernel;     /* HOST [num_conv], odd                                          */
  const int32_t *filters;    /* HOST [num_conv] output channels                               */
  const void *const *Wc;     /* HOST array of num_conv device pointers, [k, k, c_in, c_out]   */
  const void *const *bc;     /* HOST array of device pointers or NULL; NULL entry = zero bias */
  pfg_mlp dense;
} pfg_convnet;

int pfg_convnet_workspace_bytes(const pfg_convnet *net, int64_t B, size_t *bytes);

/* Per-example gradients (Section 5.3) of ell_b = -log softmax(y_b)[labels[b]] for every parameter.
 * A convolution's filter is shared by all positions of an image, so an example's filter gradient
 * is a sum over the positions (one product per example); different examples stay separate.
 *   X        [B, height, width, channels] float32
 *   dWc_out  HOST array of num_conv device pointers, entry i is [B, k, k, c_in, c_out]; NULL skips
 *   dbc_out  HOST array of num_conv device pointers, entry i is [B, c_out]; NULL skips
 *   dW_out, db_out, loss_out   for the dense layers, as for pfg_per_example_grads */
int pfg_convnet_per_example_grads(const pfg_convnet *net, const void *X, const int32_t *labels,
                                  int64_t B, float *const *dWc_out, float *const *dbc_out,
                                  float *const *dW_out, float *const *db_out, float *loss_out,
                                  void *workspace, size_t workspace_bytes, void *hip_stream);

/* Norms of the per-example gradients above without writing the gradients out.  One figure per
 * parameter block, conv blocks first: column i < num_conv is the filter of conv block i together
 * with its bias (when net->bc and net->bc[i] are non-NULL), column num_conv + l - 1 the dense layer
 * l with its bias likewise.  A dense layer's gradient is an outer product, so its norm comes from
 * the two factors as for pfg_per_example_grad_norms; a filter gradient is a sum of such products
 * over the positions (Section 5.3 with the matmul case of Section 3.4), which has no such
 * shortcut: it is formed in the workspace and its squares are summed there.
 *      sq_blocks_out[b, j] = squared norm of block j of example b's gradient
 *      norm_out[b]         = sqrt(sum_j sq_blocks_out[b, j])
 *   X, labels, loss_out   as for pfg_convnet_per_example_grads
 *   sq_blocks_out [B, num_conv + L] or NULL;  norm_out [B] or NULL (at least one is required)
 * The workspace is larger than that of the gradients by the filter and bias gradients of all
 * examples (B * k * k * c_in * c_out floats per block). */
int pfg_convnet_grad_norms_workspace_bytes(const pfg_convnet *net, int64_t B, size_t *bytes);
int pfg_convnet_per_example_grad_norms(const pfg_convnet *net, const void *X, const int32_t *labels,
                                       int64_t B, float *sq_blocks_out, float *norm_out,
                                       float *loss_out, void *workspace, size_t workspace_bytes,
                                       void *hip_stream);

/* ------------------------------------------------------------------------------------------
 * A parallel-for whose body holds a conditional (Section 3.6).  Iteration i computes
 *      t = phi_pre(pre(x_i))                 a dense network; its activation is applied after the
 *                                            last layer too
 *      c = (sum_k t[k] * cond_w[k] + cond_c > 0)
 *      r = c ? then_net(t) : else_net(t)     two dense networks with input width d_T (the output
 *                                            width of pre) and the same output width
 * The vectorised form evaluates the condition for all iterations, builds the index sets I_then and
 * I_else (each in increasing order), runs each branch on the rows of its own set only and puts
 * the results back at the rows they belong to.  Here the sets and their sizes stay on the device:
 * the first product of a branch reads its rows of t through the index set, its last product
 * stores its rows through it, and the products take their row count from device memory, so there
 * is no separate subsetting or scatter pass and no synchronisation with the host.  A branch whose
 * set is empty does no work.  When the condition does not depend on the iteration
 * (invariant_cond = 0 or 1), it is not evaluated and the chosen branch runs on all rows without
 * index sets.  All three networks must be PFG_F32.
 * ---------------------------------------------------------------------------------------- */
typedef struct {
  pfg_mlp pre;
  const void *cond_w;     /* DEVICE [d_T] float32 */
  float cond_c;
  pfg_mlp then_net;
  pfg_mlp else_net;
} pfg_cond;

#define PFG_COND_PER_ITERATION (-1)

int pfg_cond_workspace_bytes(const pfg_cond *net, int64_t n, size_t *bytes);

/*   X              [n, d_0] float32
 *   invariant_cond PFG_COND_PER_ITERATION, or 0 / 1 for a loop-invariant condition of that value
 *   R_out          [n, d_out]: every row is written by exactly one branch
 *   cond_out       [n] int32 or NULL: 1 where the then branch ran
 *   counts_out     DEVICE [2] int32 or NULL: sizes of I_then and I_else
 * n is limited to 2^24 rows. */
int pfg_cond_forward(const pfg_cond *net, const void *X, int64_t n, int invariant_cond, float *R_out,
                     int32_t *cond_out, int32_t *counts_out, void *workspace, size_t workspace_bytes,
                     void *hip_stream);

/* Per-example gradients through the conditional (the body of Section 3.6 returning the gradient of
 * its own loss, Section 5.3): iteration i computes
 *      ell_i = -log softmax(r_i)[labels[i]]          (not divided by n)
 * and its gradient with respect to every weight and bias of pre, then_net and else_net.  An
 * iteration runs one branch, so its gradient with respect to the other branch's parameters is zero
 * (those slices are written as zeros); the condition selects and passes no gradient to cond_w or
 * cond_c.  The reverse sweep reuses the index sets of the forward pass: each branch's cotangent
 * products and outer products run on the rows of its own set, read and store through it, and take
 * their row count from device memory.
 *   X, invariant_cond, cond_out, counts_out   as for pfg_cond_forward
 *   labels        [n] int32, values in [0, d_out)
 *   dW_pre_out    HOST array of pre.num_layers device pointers, entry l-1 is [n, d_{l-1}, d_l]; a NULL
 *                 array or entry skips that output.  db_pre_out likewise, entries [n, d_l]
 *   dW_then_out, db_then_out, dW_else_out, db_else_out   the same for the two branches
 *   loss_out      [n] or NULL */
int pfg_cond_grads_workspace_bytes(const pfg_cond *net, int64_t n, size_t *bytes);
int pfg_cond_per_example_grads(const pfg_cond *net, const void *X, const int32_t *labels, int64_t n,
                               int invariant_cond, float *const *dW_pre_out, float *const *db_pre_out,
                               float *const *dW_then_out, float *const *db_then_out,
                               float *const *dW_else_out, float *const *db_else_out, float *loss_out,
                               int32_t *cond_out, int32_t *counts_out, void *workspace,
                               size_t workspace_bytes, void *hip_stream);

/* Text of the last error on the calling thread ("" if none).  Valid until the next call into the
 * library from that thread. */
const char *pfg_last_error(void);

/* Per-kernel device timing, for measurement.  While enabled, every kernel the library enqueues
 * carries its own pair of HIP events, attached to the dispatch, whose timestamps are the kernel's
 * begin and end on the device.  pfg_timing_query waits for the kernels enqueued so far and
 * reports, for the kernel family called `name`, the number of launches and their summed run
 * time in milliseconds since the last reset; it returns PFG_ERR_SHAPE if no launch of that
 * family was recorded.  pfg_timing_names writes the recorded family names, separated by '\n',
 * into buf (truncated to cap bytes including the final NUL).  Do not enable timing while the
 * stream is being captured into a graph.  The switch and the totals are process-wide: the facility
 * is meant for one measuring thread; calls from several threads are safe (the switch is atomic,
 * the records are locked) but their launches are summed into the same families. */
int pfg_timing_enable(int on);
int pfg_timing_reset(void);
int pfg_timing_query(const char *name, int64_t *launches, double *total_ms);
int pfg_timing_names(char *buf, size_t cap);

/* Measurement aid: out[0 .. n) = value, written as the plainest possible stream (16-byte
 * non-temporal stores, workgroups of 256 lanes in address order), to find the rate at which the
 * device's memory absorbs writes; the outer-product kernels are priced against it.
 *   out              DEVICE, 16-byte aligned;  n a multiple of 4
 *   stores_per_lane  1, 2, 4, 8 or 16: a workgroup writes that many times 4 KiB */
int pfg_fill_reference(float *out, int64_t n, float value, int stores_per_lane, void *hip_stream);

/* Library version, major * 100 + minor. */
int pfg_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PFG_H_ */
