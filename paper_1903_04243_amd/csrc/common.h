// Internal declarations shared by the HIP sources of libpfg (not part of the public C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

namespace pfg {

// Per-kernel timing.  When timing is enabled this hands out a fresh pair of events that the
// launch attaches to the kernel dispatch itself (hipExtLaunchKernelGGL), so that their timestamps
// are the kernel's own begin and end on the device; it returns false when timing is off.
bool timing_next_events(hipEvent_t *start, hipEvent_t *stop);

#define PFG_KERNEL(kern, grid, block, smem, stream, ...)                                   \
  do {                                                                                     \
    hipEvent_t ev_start_, ev_stop_;                                                        \
    if (::pfg::timing_next_events(&ev_start_, &ev_stop_))                                  \
      hipExtLaunchKernelGGL(kern, grid, block, smem, stream, ev_start_, ev_stop_, 0,       \
                            __VA_ARGS__);                                                  \
    else                                                                                   \
      hipLaunchKernelGGL(kern, grid, block, smem, stream, __VA_ARGS__);                    \
  } while (0)

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

enum Act : int { ACT_IDENTITY = 0, ACT_RELU = 1, ACT_TANH = 2, ACT_GELU = 3 };

enum Epilogue : int {
  EPI_NONE = 0,      // C = acc
  EPI_BIAS = 1,      // C = acc + bias                      (last forward layer: logits)
  EPI_FORWARD = 2,   // z = acc + bias; C = phi(z); C2 = phi'(z)   (hidden forward layer; either of C
                     // and C2 may be null)
  EPI_MASK = 3,      // C = acc * emask[m / S, n]           (cotangent step)
  EPI_HEAD = 4,      // y = acc + bias (N <= 32, optional C = y); C2 = softmax(y) - onehot(label);
                     // loss = -log softmax(y)[label]       (last forward layer fused with the head,
                     // and optionally with the cotangent step through that layer)
  EPI_LSTM_FWD = 6,  // small-problem kernel only, W = W_h [H, 4H]: acc = h_{t-1} W_h; a workgroup takes
                     // 8 hidden units with all four of their gate columns, adds x_t W_x + b (lstm_zx)
                     // and applies the LSTM cell update of step lstm_step (writes gates, c_t, h_t)
  EPI_LSTM_BWD = 5   // columns n < n_split: C = acc.  A column n >= n_split is dh[m, k], k = n - n_split,
                     // the cotangent of the hidden state entering LSTM step lstm_step + 1; it is not
                     // stored but carried through the reverse cell update of step lstm_step at once
                     // (writes that step's dz row and the running dc).
};

// One matrix product  C[M, N] = Aeff[M, K] * Weff[K, N]  with fused prologue and epilogue.
//
// A operand.  Row m of A belongs to parallel-for iteration (b, s) = (m / S, m % S) and starts at
//     A + b * a_batch_stride + s * lda            (elements)
// a_batch_stride == 0 is a loop-invariant block shared by every b (never tiled in memory).
// If a_scale is set, Aeff[m, k] = A[m, k] * a_scale[b * ld_scale + k]  (the activation-derivative
// mask of the layer the cotangent sits at, broadcast over the seed index s).
//
// W operand.  w_kn == 1: W is [K, N] row-major (forward, a W).  w_kn == 0: W is [N, K] row-major
// and the product uses its transpose (cotangent, g W^T).
//
// a_is_f32: A holds float32 even though the product runs in bf16 (rounded when staged).
struct GemmArgs {
  const void *A;
  int64_t lda;
  int64_t a_batch_stride;
  int32_t S;
  int32_t a_is_f32;
  const float *a_scale;
  int64_t ld_scale;
  const void *W;
  int64_t ldw;
  int32_t w_kn;
  int32_t bf16;         // operands of the product: 0 float32, 1 bfloat16
  int32_t M, N, K;
  const void *bias;     // [N] in the network dtype, or nullptr
  int32_t epilogue;
  int32_t act;
  float *C;
  int64_t ldc;
  float *C2;
  const float *emask;
  int64_t ld_emask;
  int32_t streaming;    // 1: C is written once and not read again by this call
  const int32_t *labels;  // EPI_HEAD: [M]
  float *loss;            // EPI_HEAD: [M] or nullptr
  // EPI_HEAD, optional first cotangent step in the same launch (W is W_L [K, N]):
  //   head_gprev[m, i] = head_mask[m, i] * sum_j C2[m, j] * W[i, j]     for i < K
  float *head_gprev;        // [M, K] or nullptr
  const float *head_mask;   // [M, K]
  // Batched product (both operands differ from one parallel-for iteration to the next): nbatch > 1
  // runs nbatch independent products; product z uses A + z * batch_A, a_scale + z * batch_scale,
  // W + z * batch_W (float32 weights only) and C + z * batch_C (strides in elements).  EPI_NONE only.
  int32_t nbatch;
  int64_t batch_A, batch_scale, batch_W, batch_C;
  // Symmetric blocks: sym_n > 0 says that N == sym_n, M is a multiple of sym_n and every
  // sym_n x sym_n block of rows of C is a symmetric matrix.  The LDS-tiled kernel then computes only
  // the tiles on and above each block's diagonal and writes the others as their mirror images
  // (float32, EPI_NONE, sym_n a multiple of 128; other kernels ignore the hint and compute everything).
  int32_t sym_n;
  // EPI_LSTM_BWD (row m belongs to example m / S, whose gates and cell states are shared by its S rows)
  int32_t n_split;
  int32_t lstm_H, lstm_T, lstm_step;
  const float *lstm_gates;   // [B, T, 4H] gate activations i, g, f, o
  const float *lstm_cs;      // [B, T, H] cell states
  float *lstm_dc;            // [M, H] running cotangent of the cell state, updated in place
  float *lstm_dz;            // row m at lstm_dz + m * lstm_dz_ld, 4H wide: dz of step lstm_step
  int64_t lstm_dz_ld;
  // EPI_LSTM_BWD on rows chosen on the device (register-fed kernel, sub_gather set, no scatter): row m
  // of the product is iteration p = sub_rows[sub[1] + m]; its gate values and cell states are read at
  // token row lstm_zx_rows[p] + lstm_step of lstm_gates [tokens, 4H] and lstm_cs [tokens, H], lstm_dc
  // and lstm_dz are indexed by p, the same dz also goes to that token row of lstm_tok_dz (if given),
  // and lstm_seed[p, :] is added to the product where lstm_steps[p] == lstm_step + 1 (the trip is the
  // iteration's last: it enters the reverse loop here)
  float *lstm_tok_dz;
  const float *lstm_seed;
  const int32_t *lstm_steps;
  // EPI_LSTM_FWD (M rows, one per active sequence)
  const float *lstm_zx;         // x_t W_x + b, 4H wide rows; row of (m, step): lstm_zx_rows ?
  const int32_t *lstm_zx_rows;  //   lstm_zx_rows[m] + step (sequences stored back to back) : m * T + step
  float *lstm_gates_w;          // [M, T, 4H], receives step lstm_step; nullptr: gates are not kept
  float *lstm_cs_w;             // cell state of (m, step) at lstm_cs_w + m * lstm_state_ld + step * lstm_state_ts
  float *lstm_hs_w;             // hidden state, same addressing (the product's A operand is read elsewhere)
  int64_t lstm_state_ld, lstm_state_ts;   // [M, T, H] history: T * H and H; state updated in place: H and 0
  int32_t lstm_has_prev;        // 0: c_{step-1} is zero and is not read
  // history by token row (sequences stored back to back, lstm_zx_rows given): the step's gate values
  // [tokens, 4H], cell state and hidden state [tokens, H] also go to row lstm_zx_rows[m] + step of these
  // (any may be nullptr); register-fed kernel only
  float *lstm_tok_gates, *lstm_tok_c, *lstm_tok_h;
  // halting score of the new hidden state, in pieces (register-fed kernel with a row list only): the
  // workgroup that finishes hidden units 8 j .. 8 j + 7 of iteration p stores
  // sum_k h[p, k] * lstm_halt_w[k] over its units at lstm_score_part[p * lstm_score_ld + j]
  // (lstm_score_ld >= ceil(H / 8)); whoever needs the score adds the pieces in a fixed order
  const float *lstm_halt_w;
  float *lstm_score_part;
  int32_t lstm_score_ld;
  // a_km == 1: the A operand is stored transposed, [K, M] row-major with row stride lda (row k holds
  // A[0 .. M, k]); a product can then contract over the ROWS of a matrix it also uses row by row
  // elsewhere.  LDS-tiled kernel only; float32, no scale, S == 1, EPI_NONE, M a multiple of 4 and
  // 16-byte aligned rows (see akm_supported).
  int32_t a_km;
  // conv_k > 0: the A operand is the patch matrix of an image batch that is never written out.  A
  // points at the images [nbatch or B, conv_h, conv_w, conv_c] (channel fastest, conv_c a multiple
  // of 4, 16-byte aligned); the value at (row (b, y, x), column (ky, kx, c)) is
  // image[b, y + ky - p, x + kx - p, c], p = (conv_k - 1) / 2, zero outside the image.  Without a_km
  // the rows m = (b, y, x) run over all images and K = conv_k^2 conv_c; with a_km (and nbatch images,
  // image z at A + z * batch_A) the product contracts over the positions, M = conv_k^2 conv_c and
  // K = conv_h conv_w.  LDS-tiled kernel, 64 x 64 tiles, float32, FAST-load conditions on W (see
  // conv_gather_supported).
  int32_t conv_k, conv_h, conv_w, conv_c;
  // Rows chosen on the device (the index sets of a conditional, Section 3.6).  When `sub` is set the
  // product runs on rows m < sub[0] only (sub[0] <= M; M still sizes the grid).  With sub_gather, row
  // m of the A operand is row sub_rows[sub[1] + m] of A; with sub_scatter, row m of the result is
  // stored at row sub_rows[sub[1] + m] of C (and C2).  float32 operands, S == 1, no batching;
  // EPI_NONE, EPI_BIAS, EPI_FORWARD, EPI_MASK (the mask rows are those of the packed rows m) and, in
  // the small-problem kernel, EPI_LSTM_FWD.
  const int32_t *sub;           // {row count, offset into sub_rows}
  const int32_t *sub_rows;
  int32_t sub_gather, sub_scatter;
  // 1: sub[1] is 0 and sub_rows has M readable entries (the lists of a while loop): the register-fed
  // kernel then requests its list entries together with the count, not behind it
  int32_t sub_offset_zero;
  // Register-fed kernel with a row list: 0 numbers the column tiles of a row tile next to each other
  // (the live workgroups, those of the first row tiles, then come first in the launch: best when there
  // are many column tiles), 1 numbers the row tiles of a column tile next to each other (measured
  // better for the reverse trip of a while loop, 8 column tiles with a 1024-long contraction)
  int32_t sub_rows_fastest;
};

// Picks the LDS-tiled kernel or the small-problem kernel.
hipError_t launch_gemm(const GemmArgs &g, hipStream_t stream);
// May this product (with a_km set) be launched?  Alignment, sizes, and enough tiles for the
// LDS-tiled kernel, the only one that reads a transposed A.
bool akm_supported(const GemmArgs &g);
hipError_t launch_gemm_skinny(const GemmArgs &g, hipStream_t stream);
// 16 x 16 tiles for the smallest float32 products (used by launch_gemm_skinny when it applies)
// A float32 product with a contraction of 32, 64 or 128 and at least 16384 rows (plain or bias epilogue,
// W in [K, N] layout, N a multiple of 128): the kernel that keeps a W tile in LDS and streams the rows past it.
bool gemm_shortk_applies(const GemmArgs &g);
hipError_t launch_gemm_shortk(const GemmArgs &g, hipStream_t stream);
bool conv_gather_supported(const GemmArgs &g);     // may this product (conv_k > 0) be launched?
bool lstm_step_tiled_applies(const GemmArgs &g);   // EPI_LSTM_FWD on enough rows for the LDS-tiled kernel
bool small16_applies(const GemmArgs &g);
bool small16_batched_applies(const GemmArgs &g);   // a batched product (nbatch > 1) it takes in one launch
hipError_t launch_gemm_small16(const GemmArgs &g, hipStream_t stream);

// out[m, i, j] = a[m / S, i] * g[m, j]   for m < M, i < d_in, j < d_out   (float32 out)
struct OuterArgs {
  const void *a;        // [M / S, d_in], float32 or bf16
  int64_t lda;
  int32_t a_bf16;
  const float *g;       // [M, d_out]
  int64_t ldg;
  float *out;           // [M, d_in, d_out]
  int64_t M;
  int32_t S;
  int32_t d_in, d_out;
  // Iterations chosen on the device (the index sets of a conditional): when `sub` is set, M is the
  // length of the list sub_rows and grid index m a position in it; the slice written is that of row
  // sub_rows[m].  Positions offset .. offset + count - 1 ({count, offset} = sub[0], sub[1]) form the
  // job's set: position m of it multiplies row (a_gather ? sub_rows[m] : m - offset) of a by row
  // (g_gather ? sub_rows[m] : m - offset) of g; every other position gets zeros.  S must be 1.
  const int32_t *sub;
  const int32_t *sub_rows;
  int32_t a_gather, g_gather;
};

// Enqueues the n outer products in as few launches as possible (normally one).
hipError_t launch_outer(const OuterArgs *jobs, int n, hipStream_t stream);

// out[0 .. n) = value as a plain sequential stream of 16-byte non-temporal stores, stores_per_lane
// (1, 2, 4, 8 or 16) of them per lane, i.e. that many times 4 KiB per workgroup (measurement aid)
hipError_t launch_fill_reference(float *out, int64_t n, float value, int stores_per_lane, hipStream_t stream);

// delta[b, :] = softmax(y[b, :]) - onehot(labels[b]);  loss[b] = -log softmax(y[b])[labels[b]]
hipError_t launch_head_softmax_ce(const float *y, const int32_t *labels, int64_t B, int32_t n,
                                  float *delta, float *loss, hipStream_t stream);

// G[b, s, :] = pull-back of seed row (b, s) through the head.  seeds == nullptr: identity rows.
hipError_t launch_seed_rows(const float *y, const float *seeds, int64_t seed_batch_stride,
                            int64_t B, int64_t S, int32_t n, int32_t head, float *G,
                            hipStream_t stream);

// dst[c, r] = (float) src[r, c]   for an [R, C] row-major src in float32 or bf16
hipError_t launch_transpose(const void *src, int32_t src_bf16, int32_t R, int32_t C, float *dst,
                            hipStream_t stream);

// z [B, d] (pre-activations) -> a = phi(z), dphi = phi'(z), d2phi = phi''(z); any output may be null
hipError_t launch_act_from_z(const float *z, int64_t B, int32_t d, int32_t act, float *a, float *dphi,
                             float *d2phi, hipStream_t stream);

// out[(b, s), j] = in[b * in_batch_stride + s * ld_in + j] * (mask ? mask[b * ld_mask + j] : 1)
// for b < B, s < S, j < d; out row (b, s) starts at out + (b * S + s) * ld_out.  in may be float32
// or bf16 (in_bf16).
hipError_t launch_scale_rows(const void *in, int32_t in_bf16, int64_t in_batch_stride, int64_t ld_in,
                             const float *mask, int64_t ld_mask, int64_t B, int64_t S, int32_t d,
                             float *out, int64_t ld_out, hipStream_t stream);

// A product with few output tiles and a long contraction (M = B rows against a wide layer) re-reads
// its operands once per tile of the other operand and keeps few compute units busy.  Cutting the
// contraction into Z pieces, one batch entry of the tiled kernel each, gives Z times the
// workgroups on large tiles; a second kernel adds the Z partial results [Z, M, N] (float32, from
// the caller) in a fixed order and applies the epilogue.  The functions below return the Z to use,
// 1 when the product should be launched as it is.
int split_k_shape(int64_t M, int64_t N, int64_t K, int bf16);   // from the shape alone (for sizing the partials)
int split_k_factor(const GemmArgs &g);                // 1 also when an operand's alignment rules it out
hipError_t launch_gemm_split(const GemmArgs &g, int Z, float *partials, hipStream_t stream);

// The loss head of a last layer with a long contraction and few rows: Z partial products of the
// logits (batch entries of the tiled kernel, partials [Z, M, N] float32 from the caller), then one
// kernel that adds them and does what EPI_HEAD does after its product.  g as for EPI_HEAD.  The
// functions return the Z to use, 1 when the fused head should run.
int head_split_shape(int64_t M, int64_t N, int64_t K);
int head_split_pieces(const GemmArgs &g);
hipError_t launch_head_split(const GemmArgs &g, int Z, float *partials, hipStream_t stream);

// The loss head of a narrow float32 network on few rows (N <= 16 outputs, K <= 1024 inputs, at most
// 2048 rows), one workgroup per example.  g as for EPI_HEAD with C == nullptr.  mode 0: softmax
// cross-entropy (C2 = delta, loss, optional head_gprev / head_mask cotangent step).  mode 1: the N
// rows of the softmax Jacobian per example, C2 [M * N, ldc] (optional), and their pull-back through
// the layer, head_gprev [M * N, K] (optional, needs head_mask [M, K]).
bool head_rows_applies(const GemmArgs &g);
hipError_t launch_head_rows(const GemmArgs &g, int mode, hipStream_t stream);

// Squared gradient norms of the parameter blocks of a launch (at most kNormLayers per launch):
//   sq[b * ld_sq + index] = (|a[b, :]|^2 + (has_bias ? 1 : 0)) * |g[b, :]|^2       a dense layer
//   sq[b * ld_sq + index] = |a[b, :]|^2 + (g ? |g[b, :]|^2 : 0)      sum_mode: a gradient at hand
// and, if norm is given, norm[b] = sqrt(sum over the launch's layers) (the launch must then cover
// every layer).  sq may be null when norm is given.
constexpr int kNormLayers = 16;
struct NormLayer {
  const void *a;      // [B, d_in] float32 or bf16
  const float *g;     // [B, d_out]; may be null in sum_mode
  int32_t d_in, d_out;
  int32_t a_bf16, has_bias;
  int32_t index;      // column of sq
  int32_t sum_mode;   // 0: |a|^2 (+1 with a bias) x |g|^2;  1: sum a^2 + sum g^2;  2: sum a + sum g^2 (a holds partial sums of squares)
};
hipError_t launch_grad_sqnorms(const NormLayer *layers, int n, int64_t B, float *sq, int64_t ld_sq,
                               float *norm, hipStream_t stream);

// norm[b] = sqrt(sum_l sq[b * ld_sq + l]), l < L
hipError_t launch_norm_finalize(const float *sq, int64_t ld_sq, int32_t L, int64_t B, float *norm,
                                hipStream_t stream);

// out[0 .. n) = 0
hipError_t launch_fill_zero(float *out, int64_t n, hipStream_t stream);

// out[order[j], :] = (parity[j] odd ? src_odd : src_even)[j, :]   for j < rows, d columns
hipError_t launch_scatter_rows(const float *src_even, const float *src_odd, const int32_t *parity,
                               const int32_t *order, int64_t rows, int32_t d, float *out,
                               hipStream_t stream);

// LSTM cell update of step t for every (b, k): zx [B, T, 4H] holds x_t W_x + b, zh [B, 4H] holds
// h_{t-1} W_h (nullptr at the first step); writes step t of gates [B, T, 4H], cs and hs [B, T, H].
hipError_t launch_lstm_cell_forward(const float *zx, const float *zh, float *gates, float *cs,
                                    float *hs, int64_t B, int32_t H, int32_t T, int32_t t,
                                    hipStream_t stream);

// Reverse cell step t on rows m = b * S + s: reads dh (row m at dh + b * dh_batch_stride + s * H)
// and dc [rows, H] (taken as zero if first), writes dz (row m at dz + m * dz_row_stride, 4H wide)
// and dc_{t-1} in place of dc.
hipError_t launch_lstm_cell_backward(const float *dh, int64_t dh_batch_stride, float *dc, int32_t first,
                                     const float *gates, const float *cs, int64_t rows, int32_t S,
                                     int32_t H, int32_t T, int32_t t, float *dz, int64_t dz_row_stride,
                                     hipStream_t stream);

// One or two row blocks of a per-example matrix, each a sum of outer products over steps:
//   out[b * out_bs + i * d_out + j] = sum_{t < nt} a[b * a_bs + t * a_ts + i] * g[b * g_bs + t * g_ts + j]
// for i < d_in, j < d_out (float32; nt <= 0 writes zeros).  `out` of a job points at its first row.
struct OuterSumJob {
  const float *a; int64_t a_bs, a_ts;
  const float *g; int64_t g_bs, g_ts;
  int32_t nt, d_in;
  float *out;
};
hipError_t launch_outer_sum(const OuterSumJob *jobs, int njobs, int64_t B, int32_t d_out,
                            int64_t out_bs, hipStream_t stream);

// Squared norms of the per-example LSTM gradient from Gram matrices over the steps (T <= 64):
//   sq[b, 0..3] = |dW[b]|^2, |db[b]|^2, |dWout[b]|^2, |dbout[b]|^2;  norm[b] = sqrt of their sum
// X [B, T, dx], hs [B, T, H], dz [B, T, 4H], gy [B, dy]; sq and norm are optional.
constexpr int kLstmNormMaxSteps = 64;
hipError_t launch_lstm_grad_sqnorms(const float *X, const float *hs, const float *dz, const float *gy,
                                    int64_t B, int32_t T, int32_t dx, int32_t H, int32_t dy, float *sq,
                                    float *norm, hipStream_t stream);

// out[b, j] = sum_{t < T} g[b, t, j].  scratch (optional): min(B, 32768) * kSumPieces * d floats, used
// to sum long columns in pieces when there are few of them.
constexpr int kSumPieces = 8;
hipError_t launch_sum_steps(const float *g, int64_t B, int32_t T, int32_t d, float *out,
                            float *scratch, hipStream_t stream);

// Patches of a "same"-size k x k convolution over in [B, h, w, c]: P [B h w, k k c] (one row per
// output position) and / or PT [B, k k c, h w] (the same values per example with the position index
// fastest); either may be null.
hipError_t launch_im2col(const float *in, int64_t B, int32_t h, int32_t w, int32_t c, int32_t k,
                         float *P, float *PT, hipStream_t stream);

// A conv block whose outputs sum over few taps (k k c_in <= 56, a multiple of four filters, the
// filter bank and a band of the padded image in LDS): forward product + bias, relu and 2 x 2 pooling
// in one kernel that reads the image itself; pooled / which as launch_relu_pool writes them.
bool conv_relu_pool_applies(const float *in, const float *Wc, const float *bias, int64_t B, int32_t h, int32_t w,
                            int32_t ci, int32_t k, int32_t co, const float *pooled, const uint8_t *which);
hipError_t launch_conv_relu_pool(const float *in, const float *Wc, const float *bias, int64_t B, int32_t h,
                                 int32_t w, int32_t ci, int32_t k, int32_t co, float *pooled, uint8_t *which,
                                 hipStream_t stream);

// A conv block with many input channels on a small feature map (the zero-padded image of an example
// and a chunk of the filter fit in LDS; c_in a multiple of 8, c_out of 32, at most 256 positions):
// the matrix-core operands are read from the LDS image in place, no patch matrix anywhere.
//   forward:  product + bias, relu and 2 x 2 pooling in one kernel (pooled / which as launch_relu_pool
//             writes them);
//   reverse:  din [B, h, w, ci] = dz [B, h, w, co] convolved with the flipped, transposed filter (in
//             place of the patch-cotangent product and launch_col2im; c_out a multiple of 8, c_in of 32);
//   filter:   dWc [B, k k ci, co] = for each example and tap, in_shifted^T dz over the positions
//             (k = 3 or 5, c_in and c_out multiples of 32).
bool conv_direct_forward_applies(const float *in, const float *Wc, const float *bias, int64_t B, int32_t h,
                                 int32_t w, int32_t ci, int32_t k, int32_t co, const float *pooled,
                                 const uint8_t *which);
hipError_t launch_conv_direct_forward(const float *in, const float *Wc, const float *bias, int64_t B, int32_t h,
                                      int32_t w, int32_t ci, int32_t k, int32_t co, float *pooled,
                                      uint8_t *which, hipStream_t stream);
bool conv_direct_reverse_applies(const float *dz, const float *Wc, int64_t B, int32_t h, int32_t w, int32_t ci,
                                 int32_t k, int32_t co, const float *din);
hipError_t launch_conv_direct_reverse(const float *dz, const float *Wc, int64_t B, int32_t h, int32_t w,
                                      int32_t ci, int32_t k, int32_t co, float *din, hipStream_t stream);
bool conv_filter_direct_applies(const float *in, const float *dz, int64_t B, int32_t h, int32_t w, int32_t ci,
                                int32_t k, int32_t co, const float *dWc);
hipError_t launch_conv_filter_direct(const float *in, const float *dz, int64_t B, int32_t h, int32_t w,
                                     int32_t ci, int32_t k, int32_t co, float *dWc, int streaming,
                                     float *sq_part, hipStream_t stream);
// The filter gradient of a block with few input channels (k k c_in <= 64, c_out a multiple of 32, the
// padded image and 32 columns of dz within the LDS of a workgroup): the rows (tap, channel) fill one
// or two matrix-core tiles, each lane reading its shifted image value through its own offset.
bool conv_filter_rows_applies(const float *in, const float *dz, int64_t B, int32_t h, int32_t w, int32_t ci,
                              int32_t k, int32_t co, const float *dWc);
hipError_t launch_conv_filter_rows(const float *in, const float *dz, int64_t B, int32_t h, int32_t w, int32_t ci,
                                   int32_t k, int32_t co, float *dWc, int streaming, float *sq_part,
                                   hipStream_t stream);
// With sq_part set the two filter-gradient kernels store no gradient: each workgroup leaves the sum
// of the squares of its share at sq_part[b * parts + its index within the example]; parts as below.
int conv_filter_direct_parts(int32_t ci, int32_t co);
int conv_filter_rows_parts(int32_t co);

// pooled [B, h/2, w/2, c] = max over 2 x 2 windows of relu(z [B, h, w, c]); which = index 0..3 of the
// window entry that gave it
hipError_t launch_relu_pool(const float *z, int64_t B, int32_t h, int32_t w, int32_t c, float *pooled,
                            uint8_t *which, hipStream_t stream);

// dz [B, h, w, c] from the cotangent of the pooled output (relu' and the window selection applied)
hipError_t launch_unpool_mask(const float *dpooled, const float *pooled, const uint8_t *which, int64_t B,
                              int32_t h, int32_t w, int32_t c, float *dz, hipStream_t stream);

// The same in one launch with db [B, c] = sum over the positions of dz; only for the shapes and
// alignments unpool_mask_sum_applies accepts.
bool unpool_mask_sum_applies(const float *dpooled, const float *pooled, const uint8_t *which, int64_t B,
                             int32_t h, int32_t w, int32_t c, const float *dz, const float *db);
hipError_t launch_unpool_mask_sum(const float *dpooled, const float *pooled, const uint8_t *which, int64_t B,
                                  int32_t h, int32_t w, int32_t c, float *dz, float *db, hipStream_t stream);

// din [B, h, w, c] = gather of the patch cotangents dP [B h w, k k c]
hipError_t launch_col2im(const float *dP, int64_t B, int32_t h, int32_t w, int32_t c, int32_t k,
                         float *din, hipStream_t stream);

// Conditional inside the parallel-for: flags[j] = (T[j, :] . w + c0 > 0) for j < n (T has d columns,
// row stride ldt), then rows[] = the flagged row indices in increasing order followed by the others
// in increasing order, meta = {n_then, 0, n_else, n_then} (two GemmArgs::sub descriptors).
// cnt needs cond_count_groups(n) entries.  cond_out [n] (the flags) and counts_out [2] are optional.
int64_t cond_count_groups(int64_t n);
hipError_t launch_cond_partition(const float *T, int64_t ldt, int32_t n, int32_t d, const float *w,
                                 float c0, int32_t *flags, int32_t *cnt, int32_t *rows, int32_t *meta,
                                 int32_t *cond_out, int32_t *counts_out, hipStream_t stream);
// Loop-invariant condition: cond_out[j] = flag, counts_out = {n, 0} or {0, n} (both optional)
hipError_t launch_cond_invariant(int32_t n, int32_t flag, int32_t *cond_out, int32_t *counts_out,
                                 hipStream_t stream);

// rows[m] = m for m < n and meta = {n, 0, 0, n} (flag) or {0, 0, n, 0}: the index sets of a
// loop-invariant condition, for code that runs through the sets either way
hipError_t launch_cond_identity_list(int32_t *rows, int32_t *meta, int32_t n, int32_t flag, hipStream_t stream);
// out[rows[m], :] = src[gather ? rows[m] : m - sub[1], :] if position m lies in the set sub = {count,
// offset}, else 0; m < n, d columns (a packed or row-indexed block put back at the rows of its set)
hipError_t launch_cond_scatter_rows(const float *src, int64_t ld_src, int32_t gather, const int32_t *rows,
                                    const int32_t *sub, int32_t n, int32_t d, float *out, int64_t ld_out,
                                    hipStream_t stream);

// The while loop inside a parallel-for (Section 3.7), list of active iterations kept on the device.
// launch_while_init: I = 0 .. B-1, meta = {B, 0}, steps[i] = max_steps, *trips = 0 (trips optional).
// launch_while_select, trip t: on the rows of I (meta[0] of them) evaluates
//     t < length of iteration I[m]  and  c0 + <h[I[m], :], w> <= 0          (w may be null: c0 alone)
// writes the rows that go on to I_next (order kept) and their number to meta_next = {count, 0}; an
// iteration that stops gets steps[i] = t; *trips = t + 1 if any row goes on.  Token ranges come from
// seq_offsets [B + 1], cut to [0, total_tokens].  flags needs B entries, cnt while_count_entries(B).
// launch_while_state: h_out[i] = 0 if steps[i] == 0, else row i of h_even / h_odd by (steps[i] - 1) % 2.
int64_t while_count_entries(int64_t B);
hipError_t launch_while_init(int32_t *I, int32_t *meta, int32_t *steps, int32_t *trips, int32_t B,
                             int32_t max_steps, hipStream_t stream);
hipError_t launch_while_select(const int32_t *I, const int32_t *meta, int32_t t, const int32_t *seq_offsets,
                               int32_t total_tokens, const float *h, int32_t H, const float *w, float c0,
                               int32_t B, int32_t *flags, int32_t *cnt, int32_t *I_next, int32_t *meta_next,
                               int32_t *steps, int32_t *trips, hipStream_t stream,
                               const float *score_part = nullptr, int32_t score_ld = 0);
// Lists of at most this many rows can take their halting scores in pieces from the step kernel
// (GemmArgs::lstm_score_part): condition and compaction are then one launch of one workgroup.
constexpr int kWhileOneLaunchRows = 1024;
hipError_t launch_while_state(const int32_t *steps, const float *h_even, const float *h_odd, int64_t B, int32_t H,
                              float *h_out, hipStream_t stream);
// dW[b] = sum over the steps[b] trips of iteration b of [x_t, h_{t-1}]^T dz_t, db[b] = sum of dz_t (rows by
// token: iteration b starts at seq_offsets[b]; h before trip 0 is zero); dW [B, dx + H, 4H], db [B, 4H],
// either may be nullptr.  B <= 65535.
hipError_t launch_outer_sum_ragged(const float *x, int32_t dx, const float *h_tok, int32_t H, const float *dz_tok,
                                   const int32_t *seq_offsets, const int32_t *steps, int32_t total_tokens, int64_t B,
                                   float *dW, float *db, hipStream_t stream);

// Squared norms of the per-example gradients through the while loop from the rows the sweeps left by
// token (Gram identity, no gradient is formed): sq [B, 4] = |dW|^2, |db|^2, |dWout|^2, |dbout|^2 and / or
// norm [B]; at most kWhileNormMaxTrips trips per iteration are taken into account.
constexpr int kWhileNormMaxTrips = 128;
hipError_t launch_while_grad_sqnorms(const float *x, int32_t dx, const float *h_tok, int32_t H, const float *dz_tok,
                                     const int32_t *seq_offsets, const int32_t *steps, int32_t total_tokens,
                                     const float *hfin, const float *gy, int32_t dy, int64_t B, float *sq,
                                     float *norm, hipStream_t stream);

}  // namespace pfg
