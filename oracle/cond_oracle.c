/*
 * cond_oracle.c -- float64 CPU oracle for a parallel-for whose body holds a conditional.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only the test-suite, the smoke check and the
 * benchmark's CPU-baseline leg may build, load or call it.  It shares no code, header, table or
 * helper with the HIP library and neither includes the other.
 *
 * What it is: the loop that Section 3.6 starts from, executed literally.  The result of a parfor
 * is the result of running its body for every i = 0..n-1 (Section 3.3), stacked on a new leading
 * dimension (Section 4).  The body here is
 *
 *      t = phi_pre(pre(x_i))                         "pre" part: a dense network, its activation
 *                                                    applied after the last layer too
 *      c = (sum_k t[k] * w[k] + c0 > 0)              the condition of the `if`
 *      if c:  r = then_net(t)   else:  r = else_net(t)
 *
 * and the oracle runs it with an ordinary `if` inside an ordinary loop: none of the index sets,
 * subsetting or scatter of the vectorised form appear here.  When the condition is loop invariant
 * the same loop tests a flag that does not depend on i.  All arithmetic is IEEE double; OpenMP may
 * run the iterations in parallel (stateless iterations, Section 3.4).
 *
 * Dense networks: dims d_0..d_L, W_l row-major [d_{l-1}, d_l], b_l [d_l] or NULL (zero);
 * a_0 = input, z_l = a_{l-1} W_l + b_l, a_l = phi(z_l) for l < L, output z_L.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_cond_pins.py.  Nothing in this
 * file is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { CONDO_ACT_IDENTITY = 0, CONDO_ACT_RELU = 1, CONDO_ACT_TANH = 2, CONDO_ACT_GELU = 3 };

typedef struct {
  int32_t L;
  const int32_t *dims;
  const double *const *W;
  const double *const *b;    /* NULL or NULL entries: zero bias */
  int32_t act;
} condo_mlp;

typedef struct {
  const condo_mlp *pre;
  const double *w;           /* [d_T], d_T = pre->dims[pre->L] */
  double c0;
  const condo_mlp *then_net; /* input width d_T */
  const condo_mlp *else_net; /* input width d_T, same output width as then_net */
} condo_net;

static double act_value(int act, double z) {
  switch (act) {
    case CONDO_ACT_RELU: return z > 0.0 ? z : 0.0;
    case CONDO_ACT_TANH: return tanh(z);
    case CONDO_ACT_GELU: return z * 0.5 * (1.0 + erf(z / sqrt(2.0)));
    default: return z;
  }
}

static int max_width(const condo_mlp *m) {
  int w = 0;
  for (int l = 0; l <= m->L; ++l)
    if (m->dims[l] > w) w = m->dims[l];
  return w;
}

/* out = network(in); last_act: apply phi after the last layer as well */
static void mlp_forward(const condo_mlp *m, const double *in, int last_act, double *out) {
  const int wmax = max_width(m);
  double *cur = (double *)malloc(sizeof(double) * (size_t)wmax);
  double *nxt = (double *)malloc(sizeof(double) * (size_t)wmax);
  memcpy(cur, in, sizeof(double) * (size_t)m->dims[0]);
  for (int l = 1; l <= m->L; ++l) {
    const int din = m->dims[l - 1], dout = m->dims[l];
    const double *W = m->W[l - 1];
    const double *b = (m->b && m->b[l - 1]) ? m->b[l - 1] : NULL;
    for (int j = 0; j < dout; ++j) {
      double z = b ? b[j] : 0.0;
      for (int k = 0; k < din; ++k) z += cur[k] * W[(size_t)k * dout + j];
      nxt[j] = (l < m->L || last_act) ? act_value(m->act, z) : z;
    }
    double *tmp = cur; cur = nxt; nxt = tmp;
  }
  memcpy(out, cur, sizeof(double) * (size_t)m->dims[m->L]);
  free(cur);
  free(nxt);
}

/* t = phi_pre(pre(x)) */
void condo_pre(const condo_net *net, const double *x, double *t) {
  mlp_forward(net->pre, x, 1, t);
}

/* the number whose sign decides the branch */
double condo_score(const condo_net *net, const double *x) {
  const int dT = net->pre->dims[net->pre->L];
  double *t = (double *)malloc(sizeof(double) * (size_t)dT);
  condo_pre(net, x, t);
  double s = net->c0;
  for (int k = 0; k < dT; ++k) s += t[k] * net->w[k];
  free(t);
  return s;
}

/* One branch applied to one example regardless of the condition (which != 0: the then branch).
 * Used by tests to say what a row may legitimately hold when its score is within float32
 * round-off of zero. */
void condo_branch(const condo_net *net, const double *x, int which, double *r) {
  const int dT = net->pre->dims[net->pre->L];
  double *t = (double *)malloc(sizeof(double) * (size_t)dT);
  condo_pre(net, x, t);
  mlp_forward(which ? net->then_net : net->else_net, t, 0, r);
  free(t);
}

/* One iteration of the loop.  invariant < 0: the condition is computed from this iteration's t;
 * otherwise it is the loop-invariant value `invariant` (0 or 1).  Returns the condition. */
int condo_body(const condo_net *net, const double *x, int invariant, double *r) {
  const int dT = net->pre->dims[net->pre->L];
  double *t = (double *)malloc(sizeof(double) * (size_t)dT);
  condo_pre(net, x, t);
  int c;
  if (invariant < 0) {
    double s = net->c0;
    for (int k = 0; k < dT; ++k) s += t[k] * net->w[k];
    c = s > 0.0;
  } else {
    c = invariant != 0;
  }
  if (c)
    mlp_forward(net->then_net, t, 0, r);
  else
    mlp_forward(net->else_net, t, 0, r);
  free(t);
  return c;
}

/* pfor over the n rows of X [n, d_0]: R [n, d_out], cond [n] (may be NULL) */
void condo_forward(const condo_net *net, const double *X, int64_t n, int invariant, double *R,
                   int32_t *cond) {
  const int d0 = net->pre->dims[0];
  const int dout = net->then_net->dims[net->then_net->L];
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    const int c = condo_body(net, X + i * d0, invariant, R + i * dout);
    if (cond) cond[i] = c;
  }
}

/* -------------------------------------------------------------------------------------
 * Per-example gradients through the conditional (Section 5.3 applied to the body of Section 3.6):
 * iteration i computes the gradient of its own loss
 *      ell_i = -log softmax(r_i)[label_i]        (not divided by n)
 * with respect to every parameter of pre, then_net and else_net.  The iteration runs ONE branch,
 * so its gradient with respect to the other branch's parameters is zero; the condition is a
 * selection, not a differentiable function, and passes no gradient to w or c0.
 * ------------------------------------------------------------------------------------- */
static double act_deriv(int act, double z) {
  switch (act) {
    case CONDO_ACT_RELU: return z > 0.0 ? 1.0 : 0.0;
    case CONDO_ACT_TANH: { const double t = tanh(z); return 1.0 - t * t; }
    case CONDO_ACT_GELU:
      return 0.5 * (1.0 + erf(z / sqrt(2.0))) + z * exp(-0.5 * z * z) / sqrt(2.0 * 3.14159265358979323846);
    default: return 1.0;
  }
}

/* forward pass that keeps every layer: a[0] = in, z[l] = a[l-1] W_l + b_l, a[l] = phi(z[l]) for l < L
 * (and for l = L when last_act); a[L] = z[L] otherwise.  a and z hold L + 1 arrays (z[0] unused). */
static void mlp_trace(const condo_mlp *m, const double *in, int last_act, double **a, double **z) {
  memcpy(a[0], in, sizeof(double) * (size_t)m->dims[0]);
  for (int l = 1; l <= m->L; ++l) {
    const int din = m->dims[l - 1], dout = m->dims[l];
    const double *W = m->W[l - 1];
    const double *b = (m->b && m->b[l - 1]) ? m->b[l - 1] : NULL;
    for (int j = 0; j < dout; ++j) {
      double s = b ? b[j] : 0.0;
      for (int k = 0; k < din; ++k) s += a[l - 1][k] * W[(size_t)k * dout + j];
      z[l][j] = s;
      a[l][j] = (l < m->L || last_act) ? act_value(m->act, s) : s;
    }
  }
}

/* reverse pass: gout = d ell / d (output of the network); writes dW[l-1] [d_{l-1}, d_l] and
 * db[l-1] [d_l] for every layer and gin = d ell / d (input of the network) */
static void mlp_reverse(const condo_mlp *m, double *const *a, double *const *z, int last_act,
                        const double *gout, double *const *dW, double *const *db, double *gin) {
  const int wmax = max_width(m);
  double *g = (double *)malloc(sizeof(double) * (size_t)wmax);
  double *gp = (double *)malloc(sizeof(double) * (size_t)wmax);
  for (int j = 0; j < m->dims[m->L]; ++j)
    g[j] = last_act ? gout[j] * act_deriv(m->act, z[m->L][j]) : gout[j];
  for (int l = m->L; l >= 1; --l) {
    const int din = m->dims[l - 1], dout = m->dims[l];
    const double *W = m->W[l - 1];
    for (int i = 0; i < din; ++i)
      for (int j = 0; j < dout; ++j) dW[l - 1][(size_t)i * dout + j] = a[l - 1][i] * g[j];
    for (int j = 0; j < dout; ++j) db[l - 1][j] = g[j];
    for (int i = 0; i < din; ++i) {
      double s = 0.0;
      for (int j = 0; j < dout; ++j) s += g[j] * W[(size_t)i * dout + j];
      gp[i] = (l > 1) ? s * act_deriv(m->act, z[l - 1][i]) : s;
    }
    double *tmp = g; g = gp; gp = tmp;
  }
  memcpy(gin, g, sizeof(double) * (size_t)m->dims[0]);
  free(g);
  free(gp);
}

static double **alloc_layers(const condo_mlp *m) {
  double **p = (double **)malloc(sizeof(double *) * (size_t)(m->L + 1));
  for (int l = 0; l <= m->L; ++l) p[l] = (double *)calloc((size_t)m->dims[l], sizeof(double));
  return p;
}

static void free_layers(const condo_mlp *m, double **p) {
  for (int l = 0; l <= m->L; ++l) free(p[l]);
  free(p);
}

static void zero_grads(const condo_mlp *m, double *const *dW, double *const *db) {
  for (int l = 1; l <= m->L; ++l) {
    memset(dW[l - 1], 0, sizeof(double) * (size_t)m->dims[l - 1] * (size_t)m->dims[l]);
    memset(db[l - 1], 0, sizeof(double) * (size_t)m->dims[l]);
  }
}

/* One iteration: gradients of its own loss.  dW_x / db_x: one array per layer of network x, laid out
 * [d_{l-1}, d_l] and [d_l].  Returns the condition. */
int condo_body_grads(const condo_net *net, const double *x, int label, int invariant,
                     double *const *dW_pre, double *const *db_pre, double *const *dW_then,
                     double *const *db_then, double *const *dW_else, double *const *db_else,
                     double *loss) {
  const condo_mlp *pre = net->pre;
  const int dT = pre->dims[pre->L];
  double **pa = alloc_layers(pre), **pz = alloc_layers(pre);
  mlp_trace(pre, x, 1, pa, pz);
  const double *t = pa[pre->L];
  int c;
  if (invariant < 0) {
    double s = net->c0;
    for (int k = 0; k < dT; ++k) s += t[k] * net->w[k];
    c = s > 0.0;
  } else {
    c = invariant != 0;
  }
  const condo_mlp *taken = c ? net->then_net : net->else_net;
  const condo_mlp *other = c ? net->else_net : net->then_net;
  double **ba = alloc_layers(taken), **bz = alloc_layers(taken);
  mlp_trace(taken, t, 0, ba, bz);
  const int dout = taken->dims[taken->L];
  const double *r = ba[taken->L];
  /* softmax cross-entropy of this iteration's own result */
  double mx = r[0];
  for (int j = 1; j < dout; ++j) if (r[j] > mx) mx = r[j];
  double den = 0.0;
  for (int j = 0; j < dout; ++j) den += exp(r[j] - mx);
  double *g = (double *)malloc(sizeof(double) * (size_t)dout);
  for (int j = 0; j < dout; ++j) g[j] = exp(r[j] - mx) / den;
  if (loss) *loss = -log(g[label]);
  g[label] -= 1.0;
  double *gt = (double *)malloc(sizeof(double) * (size_t)dT);
  double *gx = (double *)malloc(sizeof(double) * (size_t)pre->dims[0]);
  if (c) {
    mlp_reverse(taken, ba, bz, 0, g, dW_then, db_then, gt);
    zero_grads(other, dW_else, db_else);
  } else {
    mlp_reverse(taken, ba, bz, 0, g, dW_else, db_else, gt);
    zero_grads(other, dW_then, db_then);
  }
  mlp_reverse(pre, pa, pz, 1, gt, dW_pre, db_pre, gx);
  free(g); free(gt); free(gx);
  free_layers(taken, ba); free_layers(taken, bz);
  free_layers(pre, pa); free_layers(pre, pz);
  return c;
}

/* pfor over the n rows: every output stacked on a new leading dimension (row i at offset
 * i * size of one iteration's block).  dW_x[l-1] is [n, d_{l-1}, d_l], db_x[l-1] [n, d_l]. */
void condo_per_example_grads(const condo_net *net, const double *X, const int32_t *labels, int64_t n,
                             int invariant, double *const *dW_pre, double *const *db_pre,
                             double *const *dW_then, double *const *db_then, double *const *dW_else,
                             double *const *db_else, double *loss, int32_t *cond) {
  const condo_mlp *nets[3] = {net->pre, net->then_net, net->else_net};
  double *const *dWs[3] = {dW_pre, dW_then, dW_else};
  double *const *dbs[3] = {db_pre, db_then, db_else};
  const int d0 = net->pre->dims[0];
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    double **w[3], **b[3];
    for (int q = 0; q < 3; ++q) {
      const condo_mlp *m = nets[q];
      w[q] = (double **)malloc(sizeof(double *) * (size_t)m->L);
      b[q] = (double **)malloc(sizeof(double *) * (size_t)m->L);
      for (int l = 1; l <= m->L; ++l) {
        w[q][l - 1] = dWs[q][l - 1] + (size_t)i * m->dims[l - 1] * m->dims[l];
        b[q][l - 1] = dbs[q][l - 1] + (size_t)i * m->dims[l];
      }
    }
    const int c = condo_body_grads(net, X + i * d0, labels[i], invariant, w[0], b[0], w[1], b[1], w[2], b[2],
                                   loss ? loss + i : NULL);
    if (cond) cond[i] = c;
    for (int q = 0; q < 3; ++q) { free(w[q]); free(b[q]); }
  }
}
