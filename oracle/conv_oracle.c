/*
 * conv_oracle.c -- float64 CPU oracle for per-example gradients of a small convolutional network.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only the test-suite, the smoke check and the
 * benchmark's CPU-baseline leg may build, load or call it.  It shares no code, header, table or
 * helper with the HIP library and neither includes the other.
 *
 * What it is: the paper's parallel-for executed literally (Section 3.3, Section 4) for the
 * per-example gradients of Section 5.3 on the MNIST model of the benchmarks (Section 6.1: two
 * conv-relu-maxpool blocks followed by a linear-relu-linear block; the dropout of that block is a
 * stateful random op, Section 3.8, and is left out).  A "body" handles ONE example; the "pfor"
 * driver loops over examples and stores example b at slice b.  No blocking, fusion or reordering;
 * all arithmetic is IEEE double; OpenMP runs the example index in parallel (stateless iterations,
 * Section 3.4).
 *
 * Model.  Images are [height, width, channels] (channel index fastest).  Conv block i:
 *      z[y, x, co] = bc[co] + sum_{ky, kx, ci} in[y + ky - p, x + kx - p, ci] * Wc[ky, kx, ci, co]
 *                    with p = (k - 1) / 2, k odd, zero outside the image ("same" size, stride 1)
 *      a = relu(z)   (relu'(0) := 0)
 *      out[y, x, c] = max over the 2 x 2 window (2y.., 2x..) of a     (height and width even)
 * The last block's output, flattened in (y, x, c) order, feeds dense layers
 *      z_l = a_{l-1} W_l + b_l,  a_l = relu(z_l) for l < L,  logits y = z_L
 * Per-example loss ell = -log softmax(y)[label], never divided by the batch size.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_conv_pins.py.  Nothing in this
 * file is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
  int32_t height, width, channels;
  int32_t num_conv;
  const int32_t *kernel;      /* [num_conv] odd */
  const int32_t *filters;     /* [num_conv] */
  const double *const *Wc;    /* Wc[i] is [k, k, c_in, c_out] */
  const double *const *bc;    /* bc[i] is [c_out], or NULL / NULL entry for zero */
  int32_t L;                  /* dense layers */
  const int32_t *dims;        /* [L + 1], dims[0] = flattened size of the last conv block */
  const double *const *W;     /* W[l-1] is [d_{l-1}, d_l] */
  const double *const *b;     /* or NULL */
} convo_net;

/* Geometry of block i: input hi x wi x ci, conv output the same size with co channels, pooled
 * output hi/2 x wi/2 x co. */
static void block_dims(const convo_net *net, int i, int *hi, int *wi, int *ci, int *co) {
  int h = net->height, w = net->width, c = net->channels;
  for (int j = 0; j < i; ++j) { h /= 2; w /= 2; c = net->filters[j]; }
  *hi = h; *wi = w; *ci = c; *co = net->filters[i];
}

typedef struct {
  double **in;     /* in[i]: input of conv block i  [hi, wi, ci]  (in[0] is a copy of the image) */
  double **z;      /* z[i]: conv pre-activation     [hi, wi, co] */
  int32_t **amax;  /* amax[i]: for each pooled cell, index (into z[i]) of the window's maximum */
  double *flat;    /* output of the last block, [dims[0]] */
  double **dz;     /* dense pre-activations z_l, l = 1..L */
  double **da;     /* dense activations a_l */
} tape_t;

static tape_t tape_alloc(const convo_net *net) {
  tape_t t;
  const int nc = net->num_conv;
  t.in = (double **)malloc(sizeof(double *) * (size_t)(nc + 1));
  t.z = (double **)malloc(sizeof(double *) * (size_t)(nc + 1));
  t.amax = (int32_t **)malloc(sizeof(int32_t *) * (size_t)(nc + 1));
  for (int i = 0; i < nc; ++i) {
    int hi, wi, ci, co;
    block_dims(net, i, &hi, &wi, &ci, &co);
    t.in[i] = (double *)malloc(sizeof(double) * (size_t)hi * wi * ci);
    t.z[i] = (double *)malloc(sizeof(double) * (size_t)hi * wi * co);
    t.amax[i] = (int32_t *)malloc(sizeof(int32_t) * (size_t)(hi / 2) * (wi / 2) * co);
  }
  t.flat = (double *)malloc(sizeof(double) * (size_t)net->dims[0]);
  t.dz = (double **)malloc(sizeof(double *) * (size_t)net->L);
  t.da = (double **)malloc(sizeof(double *) * (size_t)net->L);
  for (int l = 1; l <= net->L; ++l) {
    t.dz[l - 1] = (double *)malloc(sizeof(double) * (size_t)net->dims[l]);
    t.da[l - 1] = (double *)malloc(sizeof(double) * (size_t)net->dims[l]);
  }
  return t;
}

static void tape_free(const convo_net *net, tape_t t) {
  for (int i = 0; i < net->num_conv; ++i) { free(t.in[i]); free(t.z[i]); free(t.amax[i]); }
  free(t.in); free(t.z); free(t.amax); free(t.flat);
  for (int l = 1; l <= net->L; ++l) { free(t.dz[l - 1]); free(t.da[l - 1]); }
  free(t.dz); free(t.da);
}

static void forward_one(const convo_net *net, const double *x, tape_t t) {
  const int nc = net->num_conv;
  memcpy(t.in[0], x, sizeof(double) * (size_t)net->height * net->width * net->channels);
  for (int i = 0; i < nc; ++i) {
    int hi, wi, ci, co;
    block_dims(net, i, &hi, &wi, &ci, &co);
    const int k = net->kernel[i], p = (k - 1) / 2;
    const double *W = net->Wc[i];
    const double *bias = (net->bc && net->bc[i]) ? net->bc[i] : NULL;
    const double *in = t.in[i];
    for (int y = 0; y < hi; ++y)
      for (int xx = 0; xx < wi; ++xx)
        for (int o = 0; o < co; ++o) {
          double s = bias ? bias[o] : 0.0;
          for (int ky = 0; ky < k; ++ky)
            for (int kx = 0; kx < k; ++kx) {
              const int yy = y + ky - p, xs = xx + kx - p;
              if (yy < 0 || yy >= hi || xs < 0 || xs >= wi) continue;      /* zero padding */
              for (int c = 0; c < ci; ++c)
                s += in[((size_t)yy * wi + xs) * ci + c] * W[(((size_t)ky * k + kx) * ci + c) * co + o];
            }
          t.z[i][((size_t)y * wi + xx) * co + o] = s;
        }
    /* relu, then the maximum of every 2 x 2 window (the first maximum in scan order on ties) */
    const int ho = hi / 2, wo = wi / 2;
    double *out = (i + 1 < nc) ? t.in[i + 1] : t.flat;
    for (int y = 0; y < ho; ++y)
      for (int xx = 0; xx < wo; ++xx)
        for (int o = 0; o < co; ++o) {
          double best = -1.0;
          int32_t where = 0;
          for (int dy = 0; dy < 2; ++dy)
            for (int dx = 0; dx < 2; ++dx) {
              const size_t at = ((size_t)(2 * y + dy) * wi + (2 * xx + dx)) * co + o;
              const double a = t.z[i][at] > 0.0 ? t.z[i][at] : 0.0;
              if (a > best) { best = a; where = (int32_t)at; }
            }
          out[((size_t)y * wo + xx) * co + o] = best;
          t.amax[i][((size_t)y * wo + xx) * co + o] = where;
        }
  }
  const double *prev = t.flat;
  for (int l = 1; l <= net->L; ++l) {
    const int din = net->dims[l - 1], dout = net->dims[l];
    const double *W = net->W[l - 1];
    const double *bias = (net->b && net->b[l - 1]) ? net->b[l - 1] : NULL;
    for (int j = 0; j < dout; ++j) {
      double s = bias ? bias[j] : 0.0;
      for (int r = 0; r < din; ++r) s += prev[r] * W[(size_t)r * dout + j];
      t.dz[l - 1][j] = s;
      t.da[l - 1][j] = (l < net->L) ? (s > 0.0 ? s : 0.0) : s;
    }
    prev = t.da[l - 1];
  }
}

/* Logits of one image. */
void convo_forward(const convo_net *net, const double *x, double *y) {
  tape_t t = tape_alloc(net);
  forward_one(net, x, t);
  memcpy(y, t.dz[net->L - 1], sizeof(double) * (size_t)net->dims[net->L]);
  tape_free(net, t);
}

/* Output of the last conv block (what the dense layers see), [dims[0]]. */
void convo_features(const convo_net *net, const double *x, double *flat) {
  tape_t t = tape_alloc(net);
  forward_one(net, x, t);
  memcpy(flat, t.flat, sizeof(double) * (size_t)net->dims[0]);
  tape_free(net, t);
}

static void softmax(const double *y, int n, double *p) {
  double m = y[0];
  for (int j = 1; j < n; ++j) if (y[j] > m) m = y[j];
  double den = 0.0;
  for (int j = 0; j < n; ++j) { p[j] = exp(y[j] - m); den += p[j]; }
  for (int j = 0; j < n; ++j) p[j] /= den;
}

double convo_loss(const convo_net *net, const double *x, int label) {
  const int n = net->dims[net->L];
  double *y = (double *)malloc(sizeof(double) * (size_t)n);
  double *p = (double *)malloc(sizeof(double) * (size_t)n);
  convo_forward(net, x, y);
  softmax(y, n, p);
  const double loss = -log(p[label]);
  free(y); free(p);
  return loss;
}

/* Section 5.3 body: gradient of ONE example's loss with respect to every parameter.
 *   dense:  g_L = softmax(y) - onehot;  dW_l = outer(a_{l-1}, g_l), db_l = g_l,
 *           g_{l-1} = (g_l W_l^T) * relu'(z_{l-1});  the cotangent of the flattened features is g_1 W_1^T
 *   block i (last to first), given the cotangent dout of its pooled output:
 *           da[argmax of each window] = dout (other window entries get nothing), dz = da * relu'(z)
 *           dWc[ky, kx, ci, co] = sum_{y, x} in[y + ky - p, x + kx - p, ci] * dz[y, x, co]
 *           dbc[co] = sum_{y, x} dz[y, x, co]
 *           din[yy, xs, ci] = sum over (ky, kx, co) with (y, x) = (yy - ky + p, xs - kx + p) inside
 *                             of dz[y, x, co] * Wc[ky, kx, ci, co]
 * Any output may be NULL.  dWc[i] is [k, k, c_in, c_out], dbc[i] [c_out], dW[l-1] [d_{l-1}, d_l]. */
void convo_body_per_example_grads(const convo_net *net, const double *x, int label,
                                  double *const *dWc, double *const *dbc, double *const *dW,
                                  double *const *db, double *loss) {
  const int L = net->L, nc = net->num_conv, n = net->dims[L];
  tape_t t = tape_alloc(net);
  forward_one(net, x, t);
  int maxd = net->dims[0];
  for (int l = 1; l <= L; ++l) if (net->dims[l] > maxd) maxd = net->dims[l];
  double *g = (double *)malloc(sizeof(double) * (size_t)maxd);
  double *gprev = (double *)malloc(sizeof(double) * (size_t)maxd);
  softmax(t.dz[L - 1], n, g);
  if (loss) *loss = -log(g[label]);
  g[label] -= 1.0;
  for (int l = L; l >= 1; --l) {
    const int din = net->dims[l - 1], dout = net->dims[l];
    const double *W = net->W[l - 1];
    const double *ain = (l == 1) ? t.flat : t.da[l - 2];
    if (dW && dW[l - 1])
      for (int r = 0; r < din; ++r)
        for (int j = 0; j < dout; ++j) dW[l - 1][(size_t)r * dout + j] = ain[r] * g[j];
    if (db && db[l - 1])
      for (int j = 0; j < dout; ++j) db[l - 1][j] = g[j];
    for (int r = 0; r < din; ++r) {
      double s = 0.0;
      for (int j = 0; j < dout; ++j) s += g[j] * W[(size_t)r * dout + j];
      gprev[r] = (l > 1) ? (t.dz[l - 2][r] > 0.0 ? s : 0.0) : s;
    }
    double *tmp = g; g = gprev; gprev = tmp;
  }
  /* g now holds the cotangent of the flattened output of the last conv block */
  double *dout_buf = (double *)malloc(sizeof(double) * (size_t)net->dims[0]);
  memcpy(dout_buf, g, sizeof(double) * (size_t)net->dims[0]);
  for (int i = nc - 1; i >= 0; --i) {
    int hi, wi, ci, co;
    block_dims(net, i, &hi, &wi, &ci, &co);
    const int k = net->kernel[i], p = (k - 1) / 2, ho = hi / 2, wo = wi / 2;
    const double *W = net->Wc[i];
    const double *in = t.in[i];
    double *dz = (double *)calloc((size_t)hi * wi * co, sizeof(double));
    for (size_t cell = 0; cell < (size_t)ho * wo * co; ++cell) {
      const int32_t at = t.amax[i][cell];
      if (t.z[i][at] > 0.0) dz[at] = dout_buf[cell];          /* relu'(z) at the chosen entry */
    }
    if (dWc && dWc[i])
      for (int ky = 0; ky < k; ++ky)
        for (int kx = 0; kx < k; ++kx)
          for (int c = 0; c < ci; ++c)
            for (int o = 0; o < co; ++o) {
              double s = 0.0;
              for (int y = 0; y < hi; ++y)
                for (int xx = 0; xx < wi; ++xx) {
                  const int yy = y + ky - p, xs = xx + kx - p;
                  if (yy < 0 || yy >= hi || xs < 0 || xs >= wi) continue;
                  s += in[((size_t)yy * wi + xs) * ci + c] * dz[((size_t)y * wi + xx) * co + o];
                }
              dWc[i][(((size_t)ky * k + kx) * ci + c) * co + o] = s;
            }
    if (dbc && dbc[i])
      for (int o = 0; o < co; ++o) {
        double s = 0.0;
        for (int y = 0; y < hi; ++y)
          for (int xx = 0; xx < wi; ++xx) s += dz[((size_t)y * wi + xx) * co + o];
        dbc[i][o] = s;
      }
    if (i > 0) {
      double *din = (double *)calloc((size_t)hi * wi * ci, sizeof(double));
      for (int y = 0; y < hi; ++y)
        for (int xx = 0; xx < wi; ++xx)
          for (int ky = 0; ky < k; ++ky)
            for (int kx = 0; kx < k; ++kx) {
              const int yy = y + ky - p, xs = xx + kx - p;
              if (yy < 0 || yy >= hi || xs < 0 || xs >= wi) continue;
              for (int c = 0; c < ci; ++c) {
                double s = 0.0;
                for (int o = 0; o < co; ++o)
                  s += dz[((size_t)y * wi + xx) * co + o] * W[(((size_t)ky * k + kx) * ci + c) * co + o];
                din[((size_t)yy * wi + xs) * ci + c] += s;
              }
            }
      free(dout_buf);
      dout_buf = din;       /* [hi, wi, ci] = pooled output of block i - 1 */
    }
    free(dz);
  }
  free(dout_buf); free(g); free(gprev);
  tape_free(net, t);
}

/* pfor(body, B): X is [B, height, width, channels]; every output gets a leading example index. */
void convo_per_example_grads(const convo_net *net, const double *X, const int32_t *labels, int64_t B,
                             double *const *dWc, double *const *dbc, double *const *dW,
                             double *const *db, double *loss) {
  const int L = net->L, nc = net->num_conv;
  const size_t nx = (size_t)net->height * net->width * net->channels;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < B; ++i) {
    double **a = (double **)calloc((size_t)(2 * nc + 2 * L), sizeof(double *));
    double **dWci = a, **dbci = a + nc, **dWi = a + 2 * nc, **dbi = a + 2 * nc + L;
    for (int j = 0; j < nc; ++j) {
      int hi, wi, ci, co;
      block_dims(net, j, &hi, &wi, &ci, &co);
      const size_t nW = (size_t)net->kernel[j] * net->kernel[j] * ci * co;
      if (dWc && dWc[j]) dWci[j] = dWc[j] + (size_t)i * nW;
      if (dbc && dbc[j]) dbci[j] = dbc[j] + (size_t)i * co;
    }
    for (int l = 1; l <= L; ++l) {
      if (dW && dW[l - 1]) dWi[l - 1] = dW[l - 1] + (size_t)i * net->dims[l - 1] * net->dims[l];
      if (db && db[l - 1]) dbi[l - 1] = db[l - 1] + (size_t)i * net->dims[l];
    }
    convo_body_per_example_grads(net, X + (size_t)i * nx, labels[i], dWci, dbci, dWi, dbi,
                                 loss ? loss + i : NULL);
    free(a);
  }
}

/* Squared norms of one example's gradient, one figure per parameter block: column i < num_conv is
 * the filter of conv block i together with its bias (when the block has one), column num_conv + l
 * the dense layer l + 1 likewise.  The gradient is formed first and its squares are summed: the
 * definition, with no shortcut through the factors. */
void convo_body_grad_norm(const convo_net *net, const double *x, int label, double *sq, double *norm,
                          double *loss) {
  const int L = net->L, nc = net->num_conv;
  double **a = (double **)calloc((size_t)(2 * nc + 2 * L), sizeof(double *));
  size_t *cnt = (size_t *)calloc((size_t)(2 * nc + 2 * L), sizeof(size_t));
  double **dWc = a, **dbc = a + nc, **dW = a + 2 * nc, **db = a + 2 * nc + L;
  for (int i = 0; i < nc; ++i) {
    int hi, wi, ci, co;
    block_dims(net, i, &hi, &wi, &ci, &co);
    cnt[i] = (size_t)net->kernel[i] * net->kernel[i] * ci * co;
    cnt[nc + i] = (size_t)co;
  }
  for (int l = 1; l <= L; ++l) {
    cnt[2 * nc + l - 1] = (size_t)net->dims[l - 1] * net->dims[l];
    cnt[2 * nc + L + l - 1] = (size_t)net->dims[l];
  }
  for (int j = 0; j < 2 * nc + 2 * L; ++j) a[j] = (double *)malloc(sizeof(double) * cnt[j]);
  convo_body_per_example_grads(net, x, label, dWc, dbc, dW, db, loss);
  double total = 0.0;
  for (int i = 0; i < nc; ++i) {
    double s = 0.0;
    for (size_t e = 0; e < cnt[i]; ++e) s += dWc[i][e] * dWc[i][e];
    if (net->bc && net->bc[i])
      for (size_t e = 0; e < cnt[nc + i]; ++e) s += dbc[i][e] * dbc[i][e];
    if (sq) sq[i] = s;
    total += s;
  }
  for (int l = 0; l < L; ++l) {
    double s = 0.0;
    for (size_t e = 0; e < cnt[2 * nc + l]; ++e) s += dW[l][e] * dW[l][e];
    if (net->b && net->b[l])
      for (size_t e = 0; e < cnt[2 * nc + L + l]; ++e) s += db[l][e] * db[l][e];
    if (sq) sq[nc + l] = s;
    total += s;
  }
  if (norm) *norm = sqrt(total);
  for (int j = 0; j < 2 * nc + 2 * L; ++j) free(a[j]);
  free(a); free(cnt);
}

void convo_per_example_grad_norms(const convo_net *net, const double *X, const int32_t *labels,
                                  int64_t B, double *sq, double *norm, double *loss) {
  const size_t nx = (size_t)net->height * net->width * net->channels;
  const int cols = net->num_conv + net->L;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < B; ++i)
    convo_body_grad_norm(net, X + (size_t)i * nx, labels[i], sq ? sq + (size_t)cols * i : NULL,
                         norm ? norm + i : NULL, loss ? loss + i : NULL);
}
