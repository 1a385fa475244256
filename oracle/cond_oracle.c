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
