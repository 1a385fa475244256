/*
 * lstm_oracle.c -- float64 CPU oracle for per-example gradients and input Jacobians of a
 * statically unrolled single-layer LSTM with a linear readout.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only the test-suite, the smoke check and the
 * benchmark's CPU-baseline leg may build, load or call it.  It shares no code, header, table or
 * helper with the HIP library and neither includes the other.
 *
 * What it is: the paper's parallel-for executed literally (Section 3.3: the result of a parfor is
 * the result of running the body for every i = 0..n-1; Section 4: the per-iteration outputs are
 * stacked on a new leading dimension), for the LSTM model of the benchmarks (Section 6.1: a
 * single-layer unidirectional RNN on sequences of 128-dimensional vectors, state size 256;
 * Section 6.3: every example is a complete sequence of length 10; Section 6.4: the model is
 * statically unrolled to 10 steps and the Jacobian is output with respect to input).  Each use is
 * a "body" for ONE iteration and a "pfor" driver that loops over iterations and stores iteration
 * i at slice i.  No blocking, fusion or reordering; all arithmetic is IEEE double; OpenMP runs the
 * outermost iteration index in parallel, which Section 3.4 allows for stateless iterations.
 *
 * Model (the paper cites the LSTM cell but fixes no variant; this is the common cell with a
 * forget gate, no peepholes, zero initial state):
 *      u_t = [x_t, h_{t-1}]                      (length dx + H)
 *      z_t = u_t W + b                           W row-major [dx + H, 4H], column blocks i, g, f, o
 *      i = sigmoid(z_t[0:H]),  g = tanh(z_t[H:2H]),  f = sigmoid(z_t[2H:3H]),  o = sigmoid(z_t[3H:4H])
 *      c_t = f * c_{t-1} + i * g,   h_t = o * tanh(c_t),   h_0 = c_0 = 0
 *      y = h_T Wout + bout                       Wout row-major [H, dy]
 *      per-example loss  ell = -log softmax(y)[label]   (never divided by the batch size)
 * The same W is used at every step, so an example's gradient with respect to W is the sum over
 * the T steps of that step's contribution.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_lstm_pins.py (a library LSTM
 * cell, an independent autograd library, finite differences, closed forms, a hand fixture).
 * Nothing in this file is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
  int32_t dx, H, dy, T;
  const double *W;     /* [dx + H, 4H] */
  const double *b;     /* [4H] or NULL (zero) */
  const double *Wout;  /* [H, dy] */
  const double *bout;  /* [dy] or NULL (zero) */
} lstmo_net;

static double sigmoid(double v) { return 1.0 / (1.0 + exp(-v)); }

/* Everything one example's forward pass produces, kept for the reverse sweep.  Index t = 0..T-1
 * stands for step t + 1. */
typedef struct {
  double *gi, *gg, *gf, *go;   /* [T, H] gate activations */
  double *c, *h;               /* [T, H] cell and hidden state after the step */
  double *y;                   /* [dy] */
} tape_t;

static tape_t tape_alloc(const lstmo_net *net) {
  tape_t t;
  const size_t n = (size_t)net->T * net->H;
  t.gi = (double *)malloc(sizeof(double) * n);
  t.gg = (double *)malloc(sizeof(double) * n);
  t.gf = (double *)malloc(sizeof(double) * n);
  t.go = (double *)malloc(sizeof(double) * n);
  t.c = (double *)malloc(sizeof(double) * n);
  t.h = (double *)malloc(sizeof(double) * n);
  t.y = (double *)malloc(sizeof(double) * (size_t)net->dy);
  return t;
}

static void tape_free(tape_t t) {
  free(t.gi); free(t.gg); free(t.gf); free(t.go); free(t.c); free(t.h); free(t.y);
}

/* x is [T, dx]. */
static void forward_one(const lstmo_net *net, const double *x, tape_t tp) {
  const int dx = net->dx, H = net->H, T = net->T, dy = net->dy, G = 4 * net->H;
  double *z = (double *)malloc(sizeof(double) * (size_t)G);
  for (int t = 0; t < T; ++t) {
    const double *xt = x + (size_t)t * dx;
    const double *hprev = t > 0 ? tp.h + (size_t)(t - 1) * H : NULL;   /* h_0 = 0 */
    const double *cprev = t > 0 ? tp.c + (size_t)(t - 1) * H : NULL;   /* c_0 = 0 */
    for (int col = 0; col < G; ++col) {
      double s = net->b ? net->b[col] : 0.0;
      for (int r = 0; r < dx; ++r) s += xt[r] * net->W[(size_t)r * G + col];
      if (hprev)
        for (int r = 0; r < H; ++r) s += hprev[r] * net->W[(size_t)(dx + r) * G + col];
      z[col] = s;
    }
    for (int k = 0; k < H; ++k) {
      const double i = sigmoid(z[k]), g = tanh(z[H + k]), f = sigmoid(z[2 * H + k]),
                   o = sigmoid(z[3 * H + k]);
      const double c = f * (cprev ? cprev[k] : 0.0) + i * g;
      tp.gi[(size_t)t * H + k] = i;
      tp.gg[(size_t)t * H + k] = g;
      tp.gf[(size_t)t * H + k] = f;
      tp.go[(size_t)t * H + k] = o;
      tp.c[(size_t)t * H + k] = c;
      tp.h[(size_t)t * H + k] = o * tanh(c);
    }
  }
  const double *hT = tp.h + (size_t)(T - 1) * H;
  for (int j = 0; j < dy; ++j) {
    double s = net->bout ? net->bout[j] : 0.0;
    for (int k = 0; k < H; ++k) s += hT[k] * net->Wout[(size_t)k * dy + j];
    tp.y[j] = s;
  }
  free(z);
}

/* Readout y[dy] of one sequence. */
void lstmo_forward(const lstmo_net *net, const double *x, double *y) {
  tape_t tp = tape_alloc(net);
  forward_one(net, x, tp);
  memcpy(y, tp.y, sizeof(double) * (size_t)net->dy);
  tape_free(tp);
}

/* Hidden and cell states after every step, h and c are [T, H]. */
void lstmo_states(const lstmo_net *net, const double *x, double *h, double *c) {
  tape_t tp = tape_alloc(net);
  forward_one(net, x, tp);
  memcpy(h, tp.h, sizeof(double) * (size_t)net->T * net->H);
  memcpy(c, tp.c, sizeof(double) * (size_t)net->T * net->H);
  tape_free(tp);
}

static void softmax(const double *y, int n, double *p) {
  double m = y[0];
  for (int j = 1; j < n; ++j) if (y[j] > m) m = y[j];
  double den = 0.0;
  for (int j = 0; j < n; ++j) { p[j] = exp(y[j] - m); den += p[j]; }
  for (int j = 0; j < n; ++j) p[j] /= den;
}

double lstmo_loss(const lstmo_net *net, const double *x, int label) {
  double *y = (double *)malloc(sizeof(double) * (size_t)net->dy);
  double *p = (double *)malloc(sizeof(double) * (size_t)net->dy);
  lstmo_forward(net, x, y);
  softmax(y, net->dy, p);
  const double loss = -log(p[label]);
  free(y); free(p);
  return loss;
}

/* Reverse sweep of one example for one cotangent row gy of the readout (length dy).
 *   dWout = outer(h_T, gy), dbout = gy, dh_T = Wout gy, dc_T = 0
 *   for t = T..1, with tc = tanh(c_t):
 *      dc_t   += dh_t * o * (1 - tc^2)
 *      dz_o    = dh_t * tc * o (1 - o)
 *      dz_i    = dc_t * g * i (1 - i),  dz_g = dc_t * i * (1 - g^2),  dz_f = dc_t * c_{t-1} * f (1 - f)
 *      dW     += outer(u_t, dz_t),  db += dz_t            (W is shared by all steps)
 *      [dx_t, dh_{t-1}] = dz_t W^T,   dc_{t-1} = dc_t * f
 * Any of dW [dx+H, 4H], db [4H], dWout [H, dy], dbout [dy], gx [T, dx] may be NULL. */
static void backward_one(const lstmo_net *net, const double *x, tape_t tp, const double *gy,
                         double *dW, double *db, double *dWout, double *dbout, double *gx) {
  const int dx = net->dx, H = net->H, T = net->T, dy = net->dy, G = 4 * net->H;
  const double *hT = tp.h + (size_t)(T - 1) * H;
  if (dWout)
    for (int k = 0; k < H; ++k)
      for (int j = 0; j < dy; ++j) dWout[(size_t)k * dy + j] = hT[k] * gy[j];
  if (dbout)
    for (int j = 0; j < dy; ++j) dbout[j] = gy[j];
  if (dW) memset(dW, 0, sizeof(double) * (size_t)(dx + H) * G);
  if (db) memset(db, 0, sizeof(double) * (size_t)G);

  double *dh = (double *)malloc(sizeof(double) * (size_t)H);
  double *dc = (double *)malloc(sizeof(double) * (size_t)H);
  double *dz = (double *)malloc(sizeof(double) * (size_t)G);
  for (int k = 0; k < H; ++k) {
    double s = 0.0;
    for (int j = 0; j < dy; ++j) s += gy[j] * net->Wout[(size_t)k * dy + j];
    dh[k] = s;
    dc[k] = 0.0;
  }
  for (int t = T - 1; t >= 0; --t) {
    const double *xt = x + (size_t)t * dx;
    const double *hprev = t > 0 ? tp.h + (size_t)(t - 1) * H : NULL;
    const double *cprev = t > 0 ? tp.c + (size_t)(t - 1) * H : NULL;
    for (int k = 0; k < H; ++k) {
      const double i = tp.gi[(size_t)t * H + k], g = tp.gg[(size_t)t * H + k],
                   f = tp.gf[(size_t)t * H + k], o = tp.go[(size_t)t * H + k];
      const double tc = tanh(tp.c[(size_t)t * H + k]);
      const double dct = dc[k] + dh[k] * o * (1.0 - tc * tc);
      dz[3 * H + k] = dh[k] * tc * o * (1.0 - o);
      dz[k] = dct * g * i * (1.0 - i);
      dz[H + k] = dct * i * (1.0 - g * g);
      dz[2 * H + k] = dct * (cprev ? cprev[k] : 0.0) * f * (1.0 - f);
      dc[k] = dct * f;                                      /* becomes dc_{t-1} */
    }
    if (dW) {
      for (int r = 0; r < dx; ++r)
        for (int col = 0; col < G; ++col) dW[(size_t)r * G + col] += xt[r] * dz[col];
      if (hprev)
        for (int r = 0; r < H; ++r)
          for (int col = 0; col < G; ++col) dW[(size_t)(dx + r) * G + col] += hprev[r] * dz[col];
    }
    if (db)
      for (int col = 0; col < G; ++col) db[col] += dz[col];
    if (gx)
      for (int r = 0; r < dx; ++r) {
        double s = 0.0;
        for (int col = 0; col < G; ++col) s += dz[col] * net->W[(size_t)r * G + col];
        gx[(size_t)t * dx + r] = s;
      }
    for (int r = 0; r < H; ++r) {
      double s = 0.0;
      for (int col = 0; col < G; ++col) s += dz[col] * net->W[(size_t)(dx + r) * G + col];
      dh[r] = s;                                            /* becomes dh_{t-1} */
    }
  }
  free(dh); free(dc); free(dz);
}

/* Section 5.3, per-example gradients.  body(i): forward, loss, gradient of that ONE example's
 * loss with respect to W, b, Wout and bout. */
void lstmo_body_per_example_grads(const lstmo_net *net, const double *x, int label, double *dW,
                                  double *db, double *dWout, double *dbout, double *loss) {
  tape_t tp = tape_alloc(net);
  forward_one(net, x, tp);
  double *p = (double *)malloc(sizeof(double) * (size_t)net->dy);
  softmax(tp.y, net->dy, p);
  if (loss) *loss = -log(p[label]);
  p[label] -= 1.0;                                   /* d ell / d y = softmax(y) - onehot */
  backward_one(net, x, tp, p, dW, db, dWout, dbout, NULL);
  free(p);
  tape_free(tp);
}

/* pfor(body, B): X is [B, T, dx]; dW [B, dx+H, 4H], db [B, 4H], dWout [B, H, dy], dbout [B, dy],
 * loss [B]; NULL outputs are skipped. */
void lstmo_per_example_grads(const lstmo_net *net, const double *X, const int32_t *labels,
                             int64_t B, double *dW, double *db, double *dWout, double *dbout,
                             double *loss) {
  const size_t nx = (size_t)net->T * net->dx, G = 4 * (size_t)net->H;
  const size_t nW = (size_t)(net->dx + net->H) * G, nWo = (size_t)net->H * net->dy;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < B; ++i)
    lstmo_body_per_example_grads(net, X + (size_t)i * nx, labels[i], dW ? dW + (size_t)i * nW : NULL,
                                 db ? db + (size_t)i * G : NULL,
                                 dWout ? dWout + (size_t)i * nWo : NULL,
                                 dbout ? dbout + (size_t)i * net->dy : NULL, loss ? loss + i : NULL);
}

/* Section 5.1: one iteration of the Jacobian parfor is the gradient of one scalar of the output,
 * here <seed_row, y>, with respect to the whole input sequence; J_row is [T, dx]. */
/* Norms of one example's gradient (the statistic per-example clipping needs, Section 5.3): the
 * gradient itself is formed by the body above and its squares are summed, tensor by tensor:
 *   sq[0] = |dW|^2, sq[1] = |db|^2, sq[2] = |dWout|^2, sq[3] = |dbout|^2,  norm = sqrt(sum). */
void lstmo_body_grad_norm(const lstmo_net *net, const double *x, int label, double *sq, double *norm,
                          double *loss) {
  const size_t G = 4 * (size_t)net->H;
  const size_t nW = (size_t)(net->dx + net->H) * G, nWo = (size_t)net->H * net->dy;
  double *dW = (double *)malloc(sizeof(double) * nW), *db = (double *)malloc(sizeof(double) * G);
  double *dWout = (double *)malloc(sizeof(double) * nWo), *dbout = (double *)malloc(sizeof(double) * net->dy);
  lstmo_body_per_example_grads(net, x, label, dW, db, dWout, dbout, loss);
  double s[4] = {0.0, 0.0, 0.0, 0.0};
  for (size_t e = 0; e < nW; ++e) s[0] += dW[e] * dW[e];
  for (size_t e = 0; e < G; ++e) s[1] += db[e] * db[e];
  for (size_t e = 0; e < nWo; ++e) s[2] += dWout[e] * dWout[e];
  for (int e = 0; e < net->dy; ++e) s[3] += dbout[e] * dbout[e];
  if (sq) for (int k = 0; k < 4; ++k) sq[k] = s[k];
  if (norm) *norm = sqrt(s[0] + s[1] + s[2] + s[3]);
  free(dW); free(db); free(dWout); free(dbout);
}

void lstmo_per_example_grad_norms(const lstmo_net *net, const double *X, const int32_t *labels, int64_t B,
                                  double *sq, double *norm, double *loss) {
  const size_t nx = (size_t)net->T * net->dx;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < B; ++i)
    lstmo_body_grad_norm(net, X + (size_t)i * nx, labels[i], sq ? sq + 4 * i : NULL, norm ? norm + i : NULL,
                         loss ? loss + i : NULL);
}

void lstmo_body_jacobian_input_row(const lstmo_net *net, const double *x, const double *seed_row,
                                   double *J_row) {
  tape_t tp = tape_alloc(net);
  forward_one(net, x, tp);
  backward_one(net, x, tp, seed_row, NULL, NULL, NULL, NULL, J_row);
  tape_free(tp);
}

/* Nested pfor: outer over examples b, inner over seed rows s.  J is [B, S, T, dx].  seeds == NULL
 * means the identity (S must equal dy); seed_batch_stride == 0 means one [S, dy] block shared by
 * every example (loop-invariant, hence not stacked: Section 3.4). */
void lstmo_jacobian_input(const lstmo_net *net, const double *X, int64_t B, const double *seeds,
                          int64_t S, int64_t seed_batch_stride, double *J) {
  const size_t nx = (size_t)net->T * net->dx;
  const int dy = net->dy;
#pragma omp parallel for schedule(static)
  for (int64_t b = 0; b < B; ++b) {
    const double *x = X + (size_t)b * nx;
    tape_t tp = tape_alloc(net);
    forward_one(net, x, tp);
    double *e = (double *)malloc(sizeof(double) * (size_t)dy);
    for (int64_t s = 0; s < S; ++s) {
      const double *row;
      if (seeds) {
        row = seeds + (size_t)b * seed_batch_stride + (size_t)s * dy;
      } else {
        for (int j = 0; j < dy; ++j) e[j] = (j == s) ? 1.0 : 0.0;
        row = e;
      }
      backward_one(net, x, tp, row, NULL, NULL, NULL, NULL, J + ((size_t)b * S + s) * nx);
    }
    free(e);
    tape_free(tp);
  }
}

/* ---------------------------------------------------------------------------------------
 * Sequences of different lengths (Section 6.2, the auto-batching LSTM workload: every sequence is
 * iterated to its own length, inputs are not padded).  The body of the parallel-for holds a
 * sequential while loop (Section 3.7):
 *      h, c <- 0;  t <- 0
 *      while t < len_i:  h, c <- cell(x_i[t], h, c);  t <- t + 1
 *      return h, y = h Wout + bout
 * Executed literally: one sequence at a time, each to its own length.  X holds the tokens of all
 * sequences back to back ([sum of lengths, dx]); sequence i starts at row offsets[i] and has
 * offsets[i + 1] - offsets[i] >= 1 tokens (net->T is not used).  h_out is [B, H], y_out [B, dy].
 * ------------------------------------------------------------------------------------- */
void lstmo_body_varlen_forward(const lstmo_net *net, const double *x, int64_t len, double *h_out,
                               double *y_out) {
  const int dx = net->dx, H = net->H, dy = net->dy, G = 4 * net->H;
  double *h = (double *)calloc((size_t)H, sizeof(double));
  double *c = (double *)calloc((size_t)H, sizeof(double));
  double *hn = (double *)malloc(sizeof(double) * (size_t)H);
  double *z = (double *)malloc(sizeof(double) * (size_t)G);
  int64_t t = 0;
  while (t < len) {
    const double *xt = x + (size_t)t * dx;
    for (int col = 0; col < G; ++col) {
      double s = net->b ? net->b[col] : 0.0;
      for (int r = 0; r < dx; ++r) s += xt[r] * net->W[(size_t)r * G + col];
      for (int r = 0; r < H; ++r) s += h[r] * net->W[(size_t)(dx + r) * G + col];
      z[col] = s;
    }
    for (int k = 0; k < H; ++k) {
      const double i = sigmoid(z[k]), g = tanh(z[H + k]), f = sigmoid(z[2 * H + k]),
                   o = sigmoid(z[3 * H + k]);
      c[k] = f * c[k] + i * g;
      hn[k] = o * tanh(c[k]);
    }
    memcpy(h, hn, sizeof(double) * (size_t)H);
    t = t + 1;
  }
  if (h_out) memcpy(h_out, h, sizeof(double) * (size_t)H);
  if (y_out)
    for (int j = 0; j < dy; ++j) {
      double s = net->bout ? net->bout[j] : 0.0;
      for (int k = 0; k < H; ++k) s += h[k] * net->Wout[(size_t)k * dy + j];
      y_out[j] = s;
    }
  free(h); free(c); free(hn); free(z);
}

void lstmo_varlen_forward(const lstmo_net *net, const double *X, const int64_t *offsets, int64_t B,
                          double *h_out, double *y_out) {
#pragma omp parallel for schedule(dynamic)
  for (int64_t i = 0; i < B; ++i)
    lstmo_body_varlen_forward(net, X + (size_t)offsets[i] * net->dx, offsets[i + 1] - offsets[i],
                              h_out ? h_out + (size_t)i * net->H : NULL,
                              y_out ? y_out + (size_t)i * net->dy : NULL);
}

/* -------------------------------------------------------------------------------------
 * A while loop whose condition depends on the state, nested in the parallel-for (the loop nest of
 * Section 3.7, before its conversion: "parfor i: R, T = pre(i); while cond(i, R, T): R = body(i, R, T)").
 *   pre:  h = c = 0, t = 0; T = the iteration's own tokens x[0 .. len) and its length
 *   cond: t < len  and  t < max_steps  and  halt_c + sum_k h[k] * halt_w[k] <= 0
 *         (halt_w == NULL: the score is taken as halt_c alone -- pass halt_c <= 0 to leave only the
 *         length and the cap)
 *   body: (h, c) = cell(x[t], h, c); t = t + 1
 * The condition is evaluated before every trip, also the first one (with h = 0).  After the loop
 * y = h W_out + b_out; steps_out receives the number of trips the iteration made.
 * ------------------------------------------------------------------------------------- */
void lstmo_body_while_forward(const lstmo_net *net, const double *x, int64_t len, int64_t max_steps,
                              const double *halt_w, double halt_c, double *h_out, double *y_out,
                              int64_t *steps_out) {
  const int dx = net->dx, H = net->H, dy = net->dy, G = 4 * net->H;
  double *h = (double *)calloc((size_t)H, sizeof(double));
  double *c = (double *)calloc((size_t)H, sizeof(double));
  double *hn = (double *)malloc(sizeof(double) * (size_t)H);
  double *z = (double *)malloc(sizeof(double) * (size_t)G);
  int64_t t = 0;
  for (;;) {
    /* cond(i, R, T) */
    double score = halt_c;
    if (halt_w)
      for (int k = 0; k < H; ++k) score += h[k] * halt_w[k];
    if (!(t < len && t < max_steps && score <= 0.0)) break;
    /* body(i, R, T) */
    const double *xt = x + (size_t)t * dx;
    for (int col = 0; col < G; ++col) {
      double s = net->b ? net->b[col] : 0.0;
      for (int r = 0; r < dx; ++r) s += xt[r] * net->W[(size_t)r * G + col];
      for (int r = 0; r < H; ++r) s += h[r] * net->W[(size_t)(dx + r) * G + col];
      z[col] = s;
    }
    for (int k = 0; k < H; ++k) {
      const double i = sigmoid(z[k]), g = tanh(z[H + k]), f = sigmoid(z[2 * H + k]),
                   o = sigmoid(z[3 * H + k]);
      c[k] = f * c[k] + i * g;
      hn[k] = o * tanh(c[k]);
    }
    memcpy(h, hn, sizeof(double) * (size_t)H);
    t = t + 1;
  }
  if (steps_out) *steps_out = t;
  if (h_out) memcpy(h_out, h, sizeof(double) * (size_t)H);
  if (y_out)
    for (int j = 0; j < dy; ++j) {
      double s = net->bout ? net->bout[j] : 0.0;
      for (int k = 0; k < H; ++k) s += h[k] * net->Wout[(size_t)k * dy + j];
      y_out[j] = s;
    }
  free(h); free(c); free(hn); free(z);
}

void lstmo_while_forward(const lstmo_net *net, const double *X, const int64_t *offsets, int64_t B,
                         int64_t max_steps, const double *halt_w, double halt_c, double *h_out,
                         double *y_out, int64_t *steps_out) {
#pragma omp parallel for schedule(dynamic)
  for (int64_t i = 0; i < B; ++i)
    lstmo_body_while_forward(net, X + (size_t)offsets[i] * net->dx, offsets[i + 1] - offsets[i], max_steps,
                             halt_w, halt_c, h_out ? h_out + (size_t)i * net->H : NULL,
                             y_out ? y_out + (size_t)i * net->dy : NULL, steps_out ? steps_out + i : NULL);
}

/* -------------------------------------------------------------------------------------
 * Per-example gradients (Section 5.3) of a body that holds the while loop above (Section 3.7):
 *   body(i): run the loop of lstmo_body_while_forward on the iteration's own tokens (T_i trips),
 *            y = h W_out + b_out,  ell = -log softmax(y)[label],
 *            gradient of ell with respect to W, b, W_out, b_out.
 * The loop condition is a comparison: it has no derivative, and where the score is not exactly on
 * its threshold the number of trips T_i does not change under a small change of the parameters.
 * The gradient is therefore that of the T_i cell applications the loop made, taken in reverse:
 *   dW_out = outer(h, gy), db_out = gy with gy = softmax(y) - onehot;  dh = W_out gy, dc = 0
 *   for t = T_i - 1 .. 0, with tc = tanh(c_t):
 *      dc   += dh * o * (1 - tc^2)
 *      dz_o  = dh * tc * o (1 - o),  dz_i = dc * g * i (1 - i),  dz_g = dc * i (1 - g^2),
 *      dz_f  = dc * c_{t-1} * f (1 - f)
 *      dW   += outer([x_t, h_{t-1}], dz),  db += dz;   dh = dz W_h^T,  dc = dc * f
 * With T_i = 0 the state is zero: dW = 0, db = 0, dW_out = 0, db_out = gy, ell from y = b_out.
 * Any output may be NULL.
 * ------------------------------------------------------------------------------------- */
void lstmo_body_while_grads(const lstmo_net *net, const double *x, int64_t len, int64_t max_steps,
                            const double *halt_w, double halt_c, int label, double *dW, double *db,
                            double *dWout, double *dbout, double *loss, int64_t *steps_out) {
  const int dx = net->dx, H = net->H, dy = net->dy, G = 4 * net->H;
  int64_t cap = len < max_steps ? len : max_steps;
  if (cap < 0) cap = 0;
  /* what the trips leave behind for the reverse sweep; row t belongs to trip t */
  double *gi = (double *)malloc(sizeof(double) * (size_t)(cap + 1) * H);
  double *gg = (double *)malloc(sizeof(double) * (size_t)(cap + 1) * H);
  double *gf = (double *)malloc(sizeof(double) * (size_t)(cap + 1) * H);
  double *go = (double *)malloc(sizeof(double) * (size_t)(cap + 1) * H);
  double *cs = (double *)malloc(sizeof(double) * (size_t)(cap + 1) * H);
  double *hs = (double *)malloc(sizeof(double) * (size_t)(cap + 1) * H);
  double *h = (double *)calloc((size_t)H, sizeof(double));
  double *c = (double *)calloc((size_t)H, sizeof(double));
  double *z = (double *)malloc(sizeof(double) * (size_t)G);
  int64_t t = 0;
  for (;;) {
    double score = halt_c;
    if (halt_w)
      for (int k = 0; k < H; ++k) score += h[k] * halt_w[k];
    if (!(t < len && t < max_steps && score <= 0.0)) break;
    const double *xt = x + (size_t)t * dx;
    for (int col = 0; col < G; ++col) {
      double s = net->b ? net->b[col] : 0.0;
      for (int r = 0; r < dx; ++r) s += xt[r] * net->W[(size_t)r * G + col];
      for (int r = 0; r < H; ++r) s += h[r] * net->W[(size_t)(dx + r) * G + col];
      z[col] = s;
    }
    for (int k = 0; k < H; ++k) {
      const double i = sigmoid(z[k]), g = tanh(z[H + k]), f = sigmoid(z[2 * H + k]),
                   o = sigmoid(z[3 * H + k]);
      c[k] = f * c[k] + i * g;
      gi[(size_t)t * H + k] = i;
      gg[(size_t)t * H + k] = g;
      gf[(size_t)t * H + k] = f;
      go[(size_t)t * H + k] = o;
      cs[(size_t)t * H + k] = c[k];
    }
    for (int k = 0; k < H; ++k) {
      h[k] = go[(size_t)t * H + k] * tanh(c[k]);
      hs[(size_t)t * H + k] = h[k];
    }
    t = t + 1;
  }
  const int64_t T = t;
  if (steps_out) *steps_out = T;

  double *y = (double *)malloc(sizeof(double) * (size_t)dy);
  double *gy = (double *)malloc(sizeof(double) * (size_t)dy);
  for (int j = 0; j < dy; ++j) {
    double s = net->bout ? net->bout[j] : 0.0;
    for (int k = 0; k < H; ++k) s += h[k] * net->Wout[(size_t)k * dy + j];
    y[j] = s;
  }
  softmax(y, dy, gy);
  if (loss) *loss = -log(gy[label]);
  gy[label] -= 1.0;

  if (dWout)
    for (int k = 0; k < H; ++k)
      for (int j = 0; j < dy; ++j) dWout[(size_t)k * dy + j] = h[k] * gy[j];
  if (dbout)
    for (int j = 0; j < dy; ++j) dbout[j] = gy[j];
  if (dW) memset(dW, 0, sizeof(double) * (size_t)(dx + H) * G);
  if (db) memset(db, 0, sizeof(double) * (size_t)G);

  double *dh = (double *)malloc(sizeof(double) * (size_t)H);
  double *dc = (double *)calloc((size_t)H, sizeof(double));
  double *dz = (double *)malloc(sizeof(double) * (size_t)G);
  for (int k = 0; k < H; ++k) {
    double s = 0.0;
    for (int j = 0; j < dy; ++j) s += gy[j] * net->Wout[(size_t)k * dy + j];
    dh[k] = s;
  }
  for (t = T - 1; t >= 0; --t) {
    const double *xt = x + (size_t)t * dx;
    const double *hprev = t > 0 ? hs + (size_t)(t - 1) * H : NULL;
    const double *cprev = t > 0 ? cs + (size_t)(t - 1) * H : NULL;
    for (int k = 0; k < H; ++k) {
      const double i = gi[(size_t)t * H + k], g = gg[(size_t)t * H + k], f = gf[(size_t)t * H + k],
                   o = go[(size_t)t * H + k];
      const double tc = tanh(cs[(size_t)t * H + k]);
      const double dct = dc[k] + dh[k] * o * (1.0 - tc * tc);
      dz[3 * H + k] = dh[k] * tc * o * (1.0 - o);
      dz[k] = dct * g * i * (1.0 - i);
      dz[H + k] = dct * i * (1.0 - g * g);
      dz[2 * H + k] = dct * (cprev ? cprev[k] : 0.0) * f * (1.0 - f);
      dc[k] = dct * f;
    }
    if (dW) {
      for (int r = 0; r < dx; ++r)
        for (int col = 0; col < G; ++col) dW[(size_t)r * G + col] += xt[r] * dz[col];
      if (hprev)
        for (int r = 0; r < H; ++r)
          for (int col = 0; col < G; ++col) dW[(size_t)(dx + r) * G + col] += hprev[r] * dz[col];
    }
    if (db)
      for (int col = 0; col < G; ++col) db[col] += dz[col];
    for (int r = 0; r < H; ++r) {
      double s = 0.0;
      for (int col = 0; col < G; ++col) s += dz[col] * net->W[(size_t)(dx + r) * G + col];
      dh[r] = s;
    }
  }
  free(gi); free(gg); free(gf); free(go); free(cs); free(hs); free(h); free(c); free(z);
  free(y); free(gy); free(dh); free(dc); free(dz);
}

/* pfor(body, B): tokens of all sequences back to back in X, sequence i at rows offsets[i] ..
 * offsets[i + 1]; dW [B, dx+H, 4H], db [B, 4H], dWout [B, H, dy], dbout [B, dy], loss [B], steps [B]. */
void lstmo_while_per_example_grads(const lstmo_net *net, const double *X, const int64_t *offsets,
                                   const int32_t *labels, int64_t B, int64_t max_steps,
                                   const double *halt_w, double halt_c, double *dW, double *db,
                                   double *dWout, double *dbout, double *loss, int64_t *steps_out) {
  const size_t G = 4 * (size_t)net->H;
  const size_t nW = (size_t)(net->dx + net->H) * G, nWo = (size_t)net->H * net->dy;
#pragma omp parallel for schedule(dynamic)
  for (int64_t i = 0; i < B; ++i)
    lstmo_body_while_grads(net, X + (size_t)offsets[i] * net->dx, offsets[i + 1] - offsets[i], max_steps,
                           halt_w, halt_c, labels[i], dW ? dW + (size_t)i * nW : NULL,
                           db ? db + (size_t)i * G : NULL, dWout ? dWout + (size_t)i * nWo : NULL,
                           dbout ? dbout + (size_t)i * net->dy : NULL, loss ? loss + i : NULL,
                           steps_out ? steps_out + i : NULL);
}

/* -------------------------------------------------------------------------------------
 * Norms of the per-example gradients through the while loop (the quantity per-example clipping
 * needs, Section 5.3): the body forms its gradient as above and returns the sums of its squares,
 *   sq[0] = |dW|^2, sq[1] = |db|^2, sq[2] = |dWout|^2, sq[3] = |dbout|^2,  norm = sqrt of their sum.
 * Nothing is shortened: the gradient is formed in full and its entries are squared and added.
 * ------------------------------------------------------------------------------------- */
void lstmo_body_while_grad_norm(const lstmo_net *net, const double *x, int64_t len, int64_t max_steps,
                                const double *halt_w, double halt_c, int label, double *sq, double *norm,
                                double *loss, int64_t *steps_out) {
  const size_t G = 4 * (size_t)net->H;
  const size_t nW = (size_t)(net->dx + net->H) * G, nWo = (size_t)net->H * net->dy;
  double *dW = (double *)malloc(sizeof(double) * nW), *db = (double *)malloc(sizeof(double) * G);
  double *dWout = (double *)malloc(sizeof(double) * nWo), *dbout = (double *)malloc(sizeof(double) * net->dy);
  lstmo_body_while_grads(net, x, len, max_steps, halt_w, halt_c, label, dW, db, dWout, dbout, loss, steps_out);
  double s[4] = {0.0, 0.0, 0.0, 0.0};
  for (size_t e = 0; e < nW; ++e) s[0] += dW[e] * dW[e];
  for (size_t e = 0; e < G; ++e) s[1] += db[e] * db[e];
  for (size_t e = 0; e < nWo; ++e) s[2] += dWout[e] * dWout[e];
  for (int e = 0; e < net->dy; ++e) s[3] += dbout[e] * dbout[e];
  if (sq) for (int k = 0; k < 4; ++k) sq[k] = s[k];
  if (norm) *norm = sqrt(s[0] + s[1] + s[2] + s[3]);
  free(dW); free(db); free(dWout); free(dbout);
}

/* pfor(body, B): sq [B, 4], norm [B], loss [B], steps [B]; sequences as in lstmo_while_per_example_grads. */
void lstmo_while_per_example_grad_norms(const lstmo_net *net, const double *X, const int64_t *offsets,
                                        const int32_t *labels, int64_t B, int64_t max_steps,
                                        const double *halt_w, double halt_c, double *sq, double *norm,
                                        double *loss, int64_t *steps_out) {
#pragma omp parallel for schedule(dynamic)
  for (int64_t i = 0; i < B; ++i)
    lstmo_body_while_grad_norm(net, X + (size_t)offsets[i] * net->dx, offsets[i + 1] - offsets[i], max_steps,
                               halt_w, halt_c, labels[i], sq ? sq + 4 * i : NULL, norm ? norm + i : NULL,
                               loss ? loss + i : NULL, steps_out ? steps_out + i : NULL);
}
