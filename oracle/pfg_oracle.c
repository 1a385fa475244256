/*
 * pfg_oracle.c -- float64 CPU oracle for per-example gradients and Jacobians of a dense
 * feed-forward network.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only the test-suite, the smoke check and
 * the benchmark's CPU-baseline leg may build, load or call it.  It shares no code, header,
 * table or helper with the HIP library and neither includes the other.
 *
 * What it is: the paper's parallel-for, executed literally.  Section 3.3 (problem statement)
 * defines the result of a parfor as the result of running the body gamma(i) for every
 * i = 0..n-1; Section 4 defines pfor(body, n) as the per-iteration outputs stacked on a new
 * leading dimension.  Each use below is therefore written as
 *      a "body" function that handles ONE iteration (one example, or one scalar output), and
 *      a "pfor" driver that loops i = 0..n-1 and stores iteration i at slice i of the output.
 * There is no blocking, fusion, vectorisation or reordering beyond that definition.  All
 * arithmetic is IEEE double.  The only concession to run time is an OpenMP "parallel for"
 * over the outermost iteration index, which Section 3.4 explicitly allows (stateless
 * iterations may run in any order or interleaving with the same result).
 *
 * Network convention (the paper never fixes a model; these follow the workload description):
 *      dims d_0 .. d_L, W_l row-major [d_{l-1}, d_l], bias b_l [d_l] (NULL = zero)
 *      a_0 = x;  z_l = a_{l-1} W_l + b_l;  a_l = phi(z_l) for l < L;  y = z_L
 *      per-example loss  ell = -log softmax(y)[label]   (never divided by the batch size:
 *      Section 5.3 -- contributions of different examples are kept separate, not summed)
 *
 * Parity pins: every function here is pinned by tests/test_oracle_pins.py (closed forms,
 * invariants, finite differences, an independent autograd library, brute force).  Nothing in
 * this file is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define PFGO_PI 3.14159265358979323846

enum { PFGO_ACT_IDENTITY = 0, PFGO_ACT_RELU = 1, PFGO_ACT_TANH = 2, PFGO_ACT_GELU = 3 };
enum { PFGO_HEAD_LOGITS = 0, PFGO_HEAD_SOFTMAX = 1 };

typedef struct {
  int32_t L;               /* number of dense layers, >= 1                    */
  const int32_t *dims;     /* L+1 widths d_0..d_L                             */
  const double *const *W;  /* L pointers, W[l-1] is W_l, row-major [in,out]   */
  const double *const *b;  /* L pointers, b[l-1] is b_l, or NULL for zero     */
  int32_t act;             /* hidden activation phi (PFGO_ACT_*)              */
} pfgo_net;

/* ---------------------------------------------------------------------------------------
 * Activations (component-wise ops, Section 3.4: the vectorised op is the op itself).
 * ------------------------------------------------------------------------------------- */
double pfgo_act(int act, double z) {
  switch (act) {
    case PFGO_ACT_RELU: return z > 0.0 ? z : 0.0;
    case PFGO_ACT_TANH: return tanh(z);
    case PFGO_ACT_GELU: return z * 0.5 * (1.0 + erf(z / sqrt(2.0)));   /* z * Phi(z) */
    default: return z;
  }
}

double pfgo_act_deriv(int act, double z) {
  switch (act) {
    case PFGO_ACT_RELU: return z > 0.0 ? 1.0 : 0.0;                    /* phi'(0) := 0 */
    case PFGO_ACT_TANH: { double t = tanh(z); return 1.0 - t * t; }
    case PFGO_ACT_GELU: {
      double Phi = 0.5 * (1.0 + erf(z / sqrt(2.0)));
      double pdf = exp(-0.5 * z * z) / sqrt(2.0 * PFGO_PI);
      return Phi + z * pdf;
    }
    default: return 1.0;
  }
}

/* phi''(z).  ReLU and the identity are piecewise linear: 0 everywhere (the kink of ReLU at 0
 * is given 0, consistent with phi'(0) := 0).  tanh'' = -2 tanh (1 - tanh^2).
 * GELU: d/dz [Phi(z) + z pdf(z)] = pdf(z) + pdf(z) - z^2 pdf(z) = pdf(z) (2 - z^2). */
double pfgo_act_deriv2(int act, double z) {
  switch (act) {
    case PFGO_ACT_TANH: { double t = tanh(z); return -2.0 * t * (1.0 - t * t); }
    case PFGO_ACT_GELU: {
      double pdf = exp(-0.5 * z * z) / sqrt(2.0 * PFGO_PI);
      return pdf * (2.0 - z * z);
    }
    default: return 0.0;
  }
}

int pfgo_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ---------------------------------------------------------------------------------------
 * One example's forward pass.  z[l-1] and a[l-1] receive z_l and a_l (l = 1..L); a_L = z_L.
 * ------------------------------------------------------------------------------------- */
typedef struct { double **z; double **a; } pfgo_tape;

static pfgo_tape tape_alloc(const pfgo_net *net) {
  pfgo_tape t;
  t.z = (double **)malloc(sizeof(double *) * (size_t)net->L);
  t.a = (double **)malloc(sizeof(double *) * (size_t)net->L);
  for (int l = 1; l <= net->L; ++l) {
    t.z[l - 1] = (double *)malloc(sizeof(double) * (size_t)net->dims[l]);
    t.a[l - 1] = (double *)malloc(sizeof(double) * (size_t)net->dims[l]);
  }
  return t;
}

static void tape_free(const pfgo_net *net, pfgo_tape t) {
  for (int l = 1; l <= net->L; ++l) { free(t.z[l - 1]); free(t.a[l - 1]); }
  free(t.z); free(t.a);
}

static void forward_one(const pfgo_net *net, const double *x, pfgo_tape t) {
  const double *prev = x;
  for (int l = 1; l <= net->L; ++l) {
    const int din = net->dims[l - 1], dout = net->dims[l];
    const double *W = net->W[l - 1];
    const double *bias = net->b ? net->b[l - 1] : NULL;
    for (int j = 0; j < dout; ++j) {
      double s = bias ? bias[j] : 0.0;
      for (int i = 0; i < din; ++i) s += prev[i] * W[(size_t)i * dout + j];
      t.z[l - 1][j] = s;
      t.a[l - 1][j] = (l < net->L) ? pfgo_act(net->act, s) : s;
    }
    prev = t.a[l - 1];
  }
}

/* Logits of one example, y[d_L]. */
void pfgo_forward(const pfgo_net *net, const double *x, double *y) {
  pfgo_tape t = tape_alloc(net);
  forward_one(net, x, t);
  memcpy(y, t.z[net->L - 1], sizeof(double) * (size_t)net->dims[net->L]);
  tape_free(net, t);
}

/* Softmax with the maximum subtracted first. */
void pfgo_softmax(const double *y, int n, double *p) {
  double m = y[0];
  for (int j = 1; j < n; ++j) if (y[j] > m) m = y[j];
  double den = 0.0;
  for (int j = 0; j < n; ++j) { p[j] = exp(y[j] - m); den += p[j]; }
  for (int j = 0; j < n; ++j) p[j] /= den;
}

/* Softmax cross-entropy of one example. */
double pfgo_loss(const pfgo_net *net, const double *x, int label) {
  const int n = net->dims[net->L];
  double *y = (double *)malloc(sizeof(double) * (size_t)n);
  double *p = (double *)malloc(sizeof(double) * (size_t)n);
  pfgo_forward(net, x, y);
  pfgo_softmax(y, n, p);
  double loss = -log(p[label]);
  free(y); free(p);
  return loss;
}

/* ---------------------------------------------------------------------------------------
 * Reverse sweep of one example for one cotangent row g_L (length d_L), given its tape.
 *   for l = L..1:  report g_l;  g_{l-1}[i] = phi'(z_{l-1}[i]) * sum_j g_l[j] W_l[i,j]
 * g_0 (no activation below the input) is the gradient with respect to x.
 * Any of dW / db / gx may be NULL.  dW[l-1] is [d_{l-1}, d_l], db[l-1] is [d_l].
 * ------------------------------------------------------------------------------------- */
static void backward_one(const pfgo_net *net, const double *x, pfgo_tape t, const double *gL,
                         double *const *dW, double *const *db, double *gx) {
  int maxd = 0;
  for (int l = 0; l <= net->L; ++l) if (net->dims[l] > maxd) maxd = net->dims[l];
  double *g = (double *)malloc(sizeof(double) * (size_t)maxd);
  double *gprev = (double *)malloc(sizeof(double) * (size_t)maxd);
  memcpy(g, gL, sizeof(double) * (size_t)net->dims[net->L]);
  for (int l = net->L; l >= 1; --l) {
    const int din = net->dims[l - 1], dout = net->dims[l];
    const double *W = net->W[l - 1];
    const double *ain = (l == 1) ? x : t.a[l - 2];
    if (dW && dW[l - 1])
      for (int i = 0; i < din; ++i)
        for (int j = 0; j < dout; ++j) dW[l - 1][(size_t)i * dout + j] = ain[i] * g[j];
    if (db && db[l - 1])
      for (int j = 0; j < dout; ++j) db[l - 1][j] = g[j];
    if (l > 1 || gx) {
      for (int i = 0; i < din; ++i) {
        double s = 0.0;
        for (int j = 0; j < dout; ++j) s += g[j] * W[(size_t)i * dout + j];
        gprev[i] = (l > 1) ? pfgo_act_deriv(net->act, t.z[l - 2][i]) * s : s;
      }
      double *tmp = g; g = gprev; gprev = tmp;
    }
  }
  if (gx) memcpy(gx, g, sizeof(double) * (size_t)net->dims[0]);
  free(g); free(gprev);
}

/* ---------------------------------------------------------------------------------------
 * Section 5.3, per-example gradients.  body(i): forward, loss, gradients of that ONE
 * example's loss with respect to every W_l and b_l.
 * ------------------------------------------------------------------------------------- */
void pfgo_body_per_example_grads(const pfgo_net *net, const double *x, int label,
                                 double *const *dW, double *const *db, double *loss) {
  const int n = net->dims[net->L];
  pfgo_tape t = tape_alloc(net);
  forward_one(net, x, t);
  double *p = (double *)malloc(sizeof(double) * (size_t)n);
  pfgo_softmax(t.z[net->L - 1], n, p);
  if (loss) *loss = -log(p[label]);
  p[label] -= 1.0;                                  /* d ell / d y = softmax(y) - onehot */
  backward_one(net, x, t, p, dW, db, NULL);
  free(p);
  tape_free(net, t);
}

/* pfor(body, B): iteration b is written at slice b.  dW[l-1] is [B, d_{l-1}, d_l],
 * db[l-1] is [B, d_l], loss is [B]; NULL entries are skipped. */
void pfgo_per_example_grads(const pfgo_net *net, const double *X, const int32_t *labels,
                            int64_t B, double *const *dW, double *const *db, double *loss) {
  const int L = net->L;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < B; ++i) {
    double **dWi = (double **)calloc((size_t)L, sizeof(double *));
    double **dbi = (double **)calloc((size_t)L, sizeof(double *));
    for (int l = 1; l <= L; ++l) {
      if (dW && dW[l - 1]) dWi[l - 1] = dW[l - 1] + (size_t)i * net->dims[l - 1] * net->dims[l];
      if (db && db[l - 1]) dbi[l - 1] = db[l - 1] + (size_t)i * net->dims[l];
    }
    pfgo_body_per_example_grads(net, X + (size_t)i * net->dims[0], labels[i], dWi, dbi,
                                loss ? loss + i : NULL);
    free(dWi); free(dbi);
  }
}

/* ---------------------------------------------------------------------------------------
 * Section 5.1, Jacobians: a parallel-for in which each iteration is the gradient of one
 * scalar of the output.  The scalar is <seed_row, y>; with seed_row = e_s it is y[s].
 * ------------------------------------------------------------------------------------- */

/* Inner body for one example and one seed row, tape already recorded. */
static void body_row_input(const pfgo_net *net, const double *x, pfgo_tape t,
                           const double *seed_row, double *J_row) {
  backward_one(net, x, t, seed_row, NULL, NULL, J_row);
}

/* One row of the input Jacobian of one example (records its own tape). */
void pfgo_body_jacobian_input_row(const pfgo_net *net, const double *x, const double *seed_row,
                                  double *J_row) {
  pfgo_tape t = tape_alloc(net);
  forward_one(net, x, t);
  body_row_input(net, x, t, seed_row, J_row);
  tape_free(net, t);
}

/* Nested pfor: outer over examples b, inner over seed rows s.  J is [B, S, d_0].
 * seeds == NULL means the identity (S must equal d_L).  seed_batch_stride == 0 means one
 * [S, d_L] block shared by every example (loop-invariant, hence not stacked: Section 3.4);
 * otherwise example b uses seeds + b*seed_batch_stride. */
void pfgo_jacobian_input(const pfgo_net *net, const double *X, int64_t B, const double *seeds,
                         int64_t S, int64_t seed_batch_stride, double *J) {
  const int d0 = net->dims[0], dL = net->dims[net->L];
#pragma omp parallel for schedule(static)
  for (int64_t b = 0; b < B; ++b) {
    const double *x = X + (size_t)b * d0;
    pfgo_tape t = tape_alloc(net);
    forward_one(net, x, t);
    double *e = (double *)malloc(sizeof(double) * (size_t)dL);
    for (int64_t s = 0; s < S; ++s) {
      const double *row;
      if (seeds) {
        row = seeds + (size_t)b * seed_batch_stride + (size_t)s * dL;
      } else {
        for (int j = 0; j < dL; ++j) e[j] = (j == s) ? 1.0 : 0.0;
        row = e;
      }
      body_row_input(net, x, t, row, J + ((size_t)b * S + s) * d0);
    }
    free(e);
    tape_free(net, t);
  }
}

/* Cotangent row of the softmax head: d softmax(y)[k] / d y = p[k] (e_k - p). */
void pfgo_softmax_jacobian_row(const double *y, int n, int k, double *row) {
  double *p = (double *)malloc(sizeof(double) * (size_t)n);
  pfgo_softmax(y, n, p);
  for (int j = 0; j < n; ++j) row[j] = p[k] * ((j == k ? 1.0 : 0.0) - p[j]);
  free(p);
}

/* Nested pfor for the Jacobian with respect to the weights: iteration (b, k) is the gradient
 * of one scalar output of example b with respect to every W_l and b_l.
 *   head == LOGITS : scalar k is <seed row k, y_b>   (identity seeds: y_b[k])
 *   head == SOFTMAX: scalar k is <seed row k, softmax(y_b)> (identity seeds: softmax(y_b)[k])
 * JW[l-1] is [B, S, d_{l-1}, d_l], Jb[l-1] is [B, S, d_l]; NULL entries are skipped. */
void pfgo_jacobian_weights(const pfgo_net *net, const double *X, int64_t B, int head,
                           const double *seeds, int64_t S, int64_t seed_batch_stride,
                           double *const *JW, double *const *Jb) {
  const int L = net->L, d0 = net->dims[0], dL = net->dims[L];
#pragma omp parallel for schedule(static)
  for (int64_t b = 0; b < B; ++b) {
    const double *x = X + (size_t)b * d0;
    pfgo_tape t = tape_alloc(net);
    forward_one(net, x, t);
    double *row = (double *)malloc(sizeof(double) * (size_t)dL);
    double *g = (double *)malloc(sizeof(double) * (size_t)dL);
    double *srow = (double *)malloc(sizeof(double) * (size_t)dL);
    double **JWi = (double **)calloc((size_t)L, sizeof(double *));
    double **Jbi = (double **)calloc((size_t)L, sizeof(double *));
    for (int64_t k = 0; k < S; ++k) {
      if (seeds) {
        memcpy(row, seeds + (size_t)b * seed_batch_stride + (size_t)k * dL,
               sizeof(double) * (size_t)dL);
      } else {
        for (int j = 0; j < dL; ++j) row[j] = (j == k) ? 1.0 : 0.0;
      }
      if (head == PFGO_HEAD_SOFTMAX) {
        /* chain through softmax: g = sum_c row[c] * d softmax(y)[c] / d y */
        for (int j = 0; j < dL; ++j) g[j] = 0.0;
        for (int c = 0; c < dL; ++c) {
          if (row[c] == 0.0) continue;
          pfgo_softmax_jacobian_row(t.z[L - 1], dL, c, srow);
          for (int j = 0; j < dL; ++j) g[j] += row[c] * srow[j];
        }
      } else {
        memcpy(g, row, sizeof(double) * (size_t)dL);
      }
      for (int l = 1; l <= L; ++l) {
        JWi[l - 1] = (JW && JW[l - 1])
                         ? JW[l - 1] + ((size_t)b * S + k) * net->dims[l - 1] * net->dims[l] : NULL;
        Jbi[l - 1] = (Jb && Jb[l - 1]) ? Jb[l - 1] + ((size_t)b * S + k) * net->dims[l] : NULL;
      }
      backward_one(net, x, t, g, JWi, Jbi, NULL);
    }
    free(row); free(g); free(srow); free(JWi); free(Jbi);
    tape_free(net, t);
  }
}

/* ---------------------------------------------------------------------------------------
 * Per-example gradient norms (the use Section 5.3 motivates: a statistic of each example's own
 * gradient).  Written as the definition: materialise example b's gradient with the Section 5.3
 * body, then sum the squares of all of its entries.
 *   sq_layers[l-1] = sum_ij (d ell / d W_l[i,j])^2 + sum_j (d ell / d b_l[j])^2
 *   norm           = sqrt(sum_l sq_layers[l-1])
 * The bias of a layer counts only if that layer has a bias (a NULL bias is not a parameter).
 * ------------------------------------------------------------------------------------- */
void pfgo_body_grad_norm(const pfgo_net *net, const double *x, int label, double *sq_layers,
                         double *norm) {
  const int L = net->L;
  double **dW = (double **)calloc((size_t)L, sizeof(double *));
  double **db = (double **)calloc((size_t)L, sizeof(double *));
  for (int l = 1; l <= L; ++l) {
    dW[l - 1] = (double *)malloc(sizeof(double) * (size_t)net->dims[l - 1] * net->dims[l]);
    db[l - 1] = (double *)malloc(sizeof(double) * (size_t)net->dims[l]);
  }
  pfgo_body_per_example_grads(net, x, label, dW, db, NULL);
  double total = 0.0;
  for (int l = 1; l <= L; ++l) {
    const size_t nW = (size_t)net->dims[l - 1] * net->dims[l];
    double sq = 0.0;
    for (size_t e = 0; e < nW; ++e) sq += dW[l - 1][e] * dW[l - 1][e];
    if (net->b && net->b[l - 1])
      for (int j = 0; j < net->dims[l]; ++j) sq += db[l - 1][j] * db[l - 1][j];
    if (sq_layers) sq_layers[l - 1] = sq;
    total += sq;
    free(dW[l - 1]); free(db[l - 1]);
  }
  if (norm) *norm = sqrt(total);
  free(dW); free(db);
}

/* pfor(body, B): sq_layers is [B, L] (or NULL), norm is [B]. */
void pfgo_per_example_grad_norms(const pfgo_net *net, const double *X, const int32_t *labels,
                                 int64_t B, double *sq_layers, double *norm) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < B; ++i)
    pfgo_body_grad_norm(net, X + (size_t)i * net->dims[0], labels[i],
                        sq_layers ? sq_layers + (size_t)i * net->L : NULL, norm ? norm + i : NULL);
}

/* ---------------------------------------------------------------------------------------
 * Hessians as the Jacobian of a Jacobian (Section 5.1): every scalar J[s, i] of the input
 * Jacobian is differentiated once more with respect to x,
 *      H[s, i, j] = d J[s, i] / d x[j],      J[s, i] = d <seed row s, y> / d x[i].
 * The body below handles ONE seed row and ONE direction j: it carries, next to every quantity
 * of the forward pass and of the reverse sweep that computes the Jacobian row, that quantity's
 * derivative along x[j] (written with a leading "d"), by the product and chain rules:
 *   forward   a_0 = x              da_0 = e_j
 *             z_l = a_{l-1} W_l    dz_l = da_{l-1} W_l
 *             a_l = phi(z_l)       da_l = phi'(z_l) dz_l
 *   reverse   g_L = seed           dg_L = 0
 *             h_{l-1} = g_l W_l^T  dh_{l-1} = dg_l W_l^T
 *             g_{l-1} = h_{l-1} phi'(z_{l-1})
 *             dg_{l-1} = dh_{l-1} phi'(z_{l-1}) + h_{l-1} phi''(z_{l-1}) dz_{l-1}
 *   J row = h_0, so column j of this seed row's Hessian is dh_0.
 * ------------------------------------------------------------------------------------- */
void pfgo_body_hessian_input_dir(const pfgo_net *net, const double *x, const double *seed_row,
                                 int j, double *col) {
  const int L = net->L;
  pfgo_tape t = tape_alloc(net);
  forward_one(net, x, t);
  /* derivative of the forward pass along x[j] */
  double **dz = (double **)malloc(sizeof(double *) * (size_t)L);
  double **da = (double **)malloc(sizeof(double *) * (size_t)L);
  for (int l = 1; l <= L; ++l) {
    const int din = net->dims[l - 1], dout = net->dims[l];
    const double *W = net->W[l - 1];
    dz[l - 1] = (double *)malloc(sizeof(double) * (size_t)dout);
    da[l - 1] = (double *)malloc(sizeof(double) * (size_t)dout);
    for (int c = 0; c < dout; ++c) {
      double s = 0.0;
      for (int i = 0; i < din; ++i) {
        const double dprev = (l == 1) ? (i == j ? 1.0 : 0.0) : da[l - 2][i];
        s += dprev * W[(size_t)i * dout + c];
      }
      dz[l - 1][c] = s;
      da[l - 1][c] = (l < L) ? pfgo_act_deriv(net->act, t.z[l - 1][c]) * s : s;
    }
  }
  /* reverse sweep and its derivative */
  int maxd = 0;
  for (int l = 0; l <= L; ++l) if (net->dims[l] > maxd) maxd = net->dims[l];
  double *g = (double *)malloc(sizeof(double) * (size_t)maxd);
  double *dg = (double *)malloc(sizeof(double) * (size_t)maxd);
  double *gp = (double *)malloc(sizeof(double) * (size_t)maxd);
  double *dgp = (double *)malloc(sizeof(double) * (size_t)maxd);
  for (int c = 0; c < net->dims[L]; ++c) { g[c] = seed_row[c]; dg[c] = 0.0; }
  for (int l = L; l >= 1; --l) {
    const int din = net->dims[l - 1], dout = net->dims[l];
    const double *W = net->W[l - 1];
    for (int i = 0; i < din; ++i) {
      double h = 0.0, dh = 0.0;
      for (int c = 0; c < dout; ++c) {
        h += g[c] * W[(size_t)i * dout + c];
        dh += dg[c] * W[(size_t)i * dout + c];
      }
      if (l > 1) {
        const double zi = t.z[l - 2][i];
        gp[i] = h * pfgo_act_deriv(net->act, zi);
        dgp[i] = dh * pfgo_act_deriv(net->act, zi) + h * pfgo_act_deriv2(net->act, zi) * dz[l - 2][i];
      } else {
        gp[i] = h;
        dgp[i] = dh;
      }
    }
    double *tmp = g; g = gp; gp = tmp;
    tmp = dg; dg = dgp; dgp = tmp;
  }
  memcpy(col, dg, sizeof(double) * (size_t)net->dims[0]);
  for (int l = 1; l <= L; ++l) { free(dz[l - 1]); free(da[l - 1]); }
  free(dz); free(da); free(g); free(dg); free(gp); free(dgp);
  tape_free(net, t);
}

/* Nested pfor over examples b, seed rows s and directions j.  H is [B, S, d_0, d_0] with
 * H[b, s, i, j] = d J[b, s, i] / d x_b[j].  Seeds as for pfgo_jacobian_input. */
void pfgo_hessian_input(const pfgo_net *net, const double *X, int64_t B, const double *seeds,
                        int64_t S, int64_t seed_batch_stride, double *H) {
  const int d0 = net->dims[0], dL = net->dims[net->L];
#pragma omp parallel for schedule(static) collapse(2)
  for (int64_t b = 0; b < B; ++b) {
    for (int64_t s = 0; s < S; ++s) {
      const double *x = X + (size_t)b * d0;
      double *e = (double *)malloc(sizeof(double) * (size_t)dL);
      double *col = (double *)malloc(sizeof(double) * (size_t)d0);
      const double *row;
      if (seeds) {
        row = seeds + (size_t)b * seed_batch_stride + (size_t)s * dL;
      } else {
        for (int c = 0; c < dL; ++c) e[c] = (c == s) ? 1.0 : 0.0;
        row = e;
      }
      double *Hbs = H + ((size_t)b * S + s) * d0 * d0;
      for (int j = 0; j < d0; ++j) {
        pfgo_body_hessian_input_dir(net, x, row, j, col);
        for (int i = 0; i < d0; ++i) Hbs[(size_t)i * d0 + j] = col[i];
      }
      free(e); free(col);
    }
  }
}

/* ---------------------------------------------------------------------------------------
 * Section 4's worked example, as a stacking-convention check: body(i) returns
 * (a[i] + b[i], a[i] - b[i]); pfor stacks iteration i at row i.
 * ------------------------------------------------------------------------------------- */
void pfgo_pfor_add_sub(const double *a, const double *b, int64_t n, int64_t width, double *sum,
                       double *diff) {
  for (int64_t i = 0; i < n; ++i) {
    const double *ai = a + i * width, *bi = b + i * width;   /* gather row i */
    for (int64_t j = 0; j < width; ++j) {
      sum[i * width + j] = ai[j] + bi[j];
      diff[i * width + j] = ai[j] - bi[j];
    }
  }
}
