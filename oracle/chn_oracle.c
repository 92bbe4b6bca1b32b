/*
 * chn_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, obviously-correct CPU statement of every array operation that
 * a define-by-run training step issues to the NumPy-like GPU array layer the
 * paper describes (Section "GPU Support by CuPy"): broadcasting element-wise
 * kernels, axis reductions, dense matrix products, plus the textbook layer
 * functions a training step needs (LSTM cell, softmax cross-entropy, SGD,
 * embedding lookup).
 *
 * Rules this file keeps:
 *   - every value is an IEEE double; callers hand in the exact fp32 / bf16
 *     input values widened to double, results stay double;
 *   - natural index order, one loop nest per definition, no blocking, no
 *     fusion, no reordering; the only parallelism is an OpenMP "parallel for"
 *     over the outermost loop of a definition;
 *   - it shares no code, header, table or constant with the HIP library and is
 *     only ever called from tests, the smoke check and the benchmark's
 *     cpu_baseline leg.
 *
 * Arrays are described the NumPy way: shape plus BYTE strides, so a transposed
 * or broadcast (stride 0) view gives the same numbers as its materialised copy.
 *
 * Parity pins (tests/test_oracle_*.py): values the paper prints (the [1,2]
 * Euclidean-norm figure, the x*y+z user kernel figure), central finite
 * differences for every backward, exact small-integer cases, closed forms,
 * invariants, and NumPy/SciPy special cases.  No function here is unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_MAX_NDIM 8

typedef struct {
  double *data;
  int32_t ndim;
  int64_t shape[ORC_MAX_NDIM];
  int64_t strides[ORC_MAX_NDIM]; /* bytes */
} orc_view;

/* element-wise operation codes (private to the oracle; the Python wrapper maps names) */
enum {
  ORC_COPY = 0,
  ORC_ADD,
  ORC_SUB,
  ORC_MUL,
  ORC_MAD,       /* x*y + z : the user-kernel figure ("my_mad") */
  ORC_MAD_RELU,  /* max(0, x*y + z) */
  ORC_RELU,      /* max(0, x) */
  ORC_RELU_BWD,  /* gy * [y > 0]        (uses the OUTPUT y, function-wise memory reduction) */
  ORC_GELU,      /* 0.5 x (1 + erf(x / sqrt 2)) */
  ORC_GELU_BWD,  /* gy * (Phi(z) + z phi(z)) */
  ORC_SCALE,     /* s0 * x */
  ORC_AXPY,      /* x + s0 * y */
  ORC_ADD_RELU,  /* max(0, x + y) */
  ORC_ADD_GELU,  /* gelu(x + y) */
  ORC_FILL,      /* s0 */
  ORC_SIGMOID,
  ORC_TANH,
  ORC_SQRT,
  ORC_EXP,
  ORC_GELU_BWD2, /* g * gelu''(z), gelu''(z) = phi(z) (2 - z^2): the derivative of Phi(z) + z phi(z) */
  ORC_N_OPS
};

static const int orc_arity[ORC_N_OPS] = {1, 2, 2, 2, 3, 3, 1, 2, 1, 2, 1, 2, 2, 2, 0, 1, 1, 1, 1, 2};

static double orc_gelu(double x) { return 0.5 * x * (1.0 + erf(x / sqrt(2.0))); }

static double orc_gelu_grad(double x) {
  const double pi = 3.14159265358979323846;
  double Phi = 0.5 * (1.0 + erf(x / sqrt(2.0)));
  double phi = exp(-0.5 * x * x) / sqrt(2.0 * pi);
  return Phi + x * phi;
}

static double orc_sigmoid(double x) { return 1.0 / (1.0 + exp(-x)); }

static double orc_apply(int op, const double *x, const double *s) {
  switch (op) {
    case ORC_COPY: return x[0];
    case ORC_ADD: return x[0] + x[1];
    case ORC_SUB: return x[0] - x[1];
    case ORC_MUL: return x[0] * x[1];
    case ORC_MAD: return x[0] * x[1] + x[2];
    case ORC_MAD_RELU: { double v = x[0] * x[1] + x[2]; return v > 0.0 ? v : 0.0; }
    case ORC_RELU: return x[0] > 0.0 ? x[0] : 0.0;
    case ORC_RELU_BWD: return x[1] > 0.0 ? x[0] : 0.0;
    case ORC_GELU: return orc_gelu(x[0]);
    case ORC_GELU_BWD: return x[0] * orc_gelu_grad(x[1]);
    case ORC_SCALE: return s[0] * x[0];
    case ORC_AXPY: return x[0] + s[0] * x[1];
    case ORC_ADD_RELU: { double v = x[0] + x[1]; return v > 0.0 ? v : 0.0; }
    case ORC_ADD_GELU: return orc_gelu(x[0] + x[1]);
    case ORC_FILL: return s[0];
    case ORC_SIGMOID: return orc_sigmoid(x[0]);
    case ORC_TANH: return tanh(x[0]);
    case ORC_SQRT: return sqrt(x[0]);
    case ORC_EXP: return exp(x[0]);
    case ORC_GELU_BWD2: return x[0] * (exp(-0.5 * x[1] * x[1]) / sqrt(2.0 * 3.14159265358979323846)) * (2.0 - x[1] * x[1]);
  }
  return NAN;
}

/* Address of the element of v that the NumPy broadcasting rule pairs with output index idx:
 * shapes are right-aligned, a size-1 dimension repeats its single element. */
static double *orc_at(const orc_view *v, const int64_t *idx, int out_ndim) {
  int64_t off = 0;
  for (int d = 0; d < v->ndim; ++d) {
    int od = out_ndim - v->ndim + d;
    int64_t i = (v->shape[d] == 1) ? 0 : idx[od];
    off += i * v->strides[d];
  }
  return (double *)((char *)v->data + off);
}

/* Broadcasting element-wise map (Section "Custom CUDA Kernels": the element-wise kernel applies
 * one operation to all elements; the array layer follows NumPy broadcasting).
 * Returns 0, or -1 when an input cannot be broadcast to the output shape. */
int orc_elementwise(int op, int n_in, const orc_view *const *in, const orc_view *out,
                    const double *scalars) {
  if (op < 0 || op >= ORC_N_OPS || n_in != orc_arity[op]) return -1;
  int nd = out->ndim;
  for (int k = 0; k < n_in; ++k) {
    if (in[k]->ndim > nd) return -1;
    for (int d = 0; d < in[k]->ndim; ++d) {
      int od = nd - in[k]->ndim + d;
      if (in[k]->shape[d] != 1 && in[k]->shape[d] != out->shape[od]) return -1;
    }
  }
  int64_t total = 1;
  for (int d = 0; d < nd; ++d) total *= out->shape[d];
  if (total == 0) return 0;
  int64_t outer = nd > 0 ? out->shape[0] : 1;
  int64_t inner = total / outer;
#pragma omp parallel for schedule(static)
  for (int64_t o = 0; o < outer; ++o) {
    int64_t idx[ORC_MAX_NDIM] = {0};
    double x[3];
    for (int64_t r = 0; r < inner; ++r) {
      /* index of this element: dimension 0 is o, the rest is r written in mixed radix */
      int64_t rem = r;
      for (int d = nd - 1; d >= 1; --d) { idx[d] = rem % out->shape[d]; rem /= out->shape[d]; }
      if (nd > 0) idx[0] = o;
      for (int k = 0; k < n_in; ++k) x[k] = *orc_at(in[k], idx, nd);
      *orc_at(out, idx, nd) = orc_apply(op, x, scalars);
    }
  }
  return 0;
}

/* Reduction over one axis (Section "Custom CUDA Kernels": the reduction kernel folds elements by a
 * binary operator; "sum" folds by +).  op 0 = sum, 1 = max.  out has the input's shape with the
 * axis removed (keepdims = 0) or set to 1 (keepdims = 1).  An empty axis gives the identity
 * (0 for sum, -inf for max). */
int orc_reduce_axis(int op, const orc_view *in, int axis, int keepdims, const orc_view *out) {
  int nd = in->ndim;
  if (axis < 0) axis += nd;
  if (axis < 0 || axis >= nd) return -1;
  int ond = keepdims ? nd : nd - 1;
  if (out->ndim != ond) return -1;
  int64_t total_out = 1;
  for (int d = 0, od = 0; d < nd; ++d) {
    if (d == axis) {
      if (keepdims) { if (out->shape[od] != 1) return -1; ++od; }
      continue;
    }
    if (out->shape[od] != in->shape[d]) return -1;
    total_out *= in->shape[d];
    ++od;
  }
  int64_t len = in->shape[axis];
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < total_out; ++r) {
    int64_t idx[ORC_MAX_NDIM] = {0};
    int64_t oidx[ORC_MAX_NDIM] = {0};
    int64_t rem = r;
    for (int d = nd - 1; d >= 0; --d) {
      if (d == axis) continue;
      idx[d] = rem % in->shape[d];
      rem /= in->shape[d];
    }
    for (int d = 0, od = 0; d < nd; ++d) {
      if (d == axis) { if (keepdims) oidx[od++] = 0; continue; }
      oidx[od++] = idx[d];
    }
    double acc = (op == 0) ? 0.0 : -INFINITY;
    for (int64_t j = 0; j < len; ++j) {
      idx[axis] = j;
      double v = *orc_at(in, idx, nd);
      if (op == 0) acc += v; else if (v > acc) acc = v;
    }
    *orc_at(out, oidx, ond) = acc;
  }
  return 0;
}

/* Dense product out[m,n] = alpha * sum_k A[m,k] B[k,n] + beta * C[m,n]
 * (the "x @ W.T" of the fully connected layer in the model-definition figure is this with
 * B a transposed view).  A (M,K), B (K,N), C and out (M,N) are 2-d views; C may be NULL when beta = 0. */
int orc_gemm(const orc_view *A, const orc_view *B, const orc_view *C, double alpha, double beta,
             const orc_view *out) {
  if (A->ndim != 2 || B->ndim != 2 || out->ndim != 2) return -1;
  int64_t M = A->shape[0], K = A->shape[1], N = B->shape[1];
  if (B->shape[0] != K || out->shape[0] != M || out->shape[1] != N) return -1;
  if (C && (C->ndim != 2 || C->shape[0] != M || C->shape[1] != N)) return -1;
  if (!C && beta != 0.0) return -1;
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m) {
    for (int64_t n = 0; n < N; ++n) {
      double acc = 0.0;
      for (int64_t k = 0; k < K; ++k) {
        double a = *(double *)((char *)A->data + m * A->strides[0] + k * A->strides[1]);
        double b = *(double *)((char *)B->data + k * B->strides[0] + n * B->strides[1]);
        acc += a * b;
      }
      double v = alpha * acc;
      if (C) v += beta * *(double *)((char *)C->data + m * C->strides[0] + n * C->strides[1]);
      *(double *)((char *)out->data + m * out->strides[0] + n * out->strides[1]) = v;
    }
  }
  return 0;
}

/* One entry of the same product, for spot checks at sizes where the full product is too slow. */
double orc_gemm_entry(const orc_view *A, const orc_view *B, int64_t m, int64_t n) {
  int64_t K = A->shape[1];
  double acc = 0.0;
  for (int64_t k = 0; k < K; ++k) {
    double a = *(double *)((char *)A->data + m * A->strides[0] + k * A->strides[1]);
    double b = *(double *)((char *)B->data + k * B->strides[0] + n * B->strides[1]);
    acc += a * b;
  }
  return acc;
}

/* LSTM cell, textbook form without peepholes.  z (B,4H) holds the gate pre-activations
 * x W + h U (bias added here when given), gate blocks along the 4H axis in the order i, f, g, o.
 *   i = sigma(z_i)  f = sigma(z_f)  g = tanh(z_g)  o = sigma(z_o)
 *   c = f * c_prev + i * g          h = o * tanh(c)
 * All arrays contiguous row-major.  gates (B,4H) receives the activated i,f,g,o. */
void orc_lstm_fwd(const double *z, const double *bias, const double *c_prev, int64_t B, int64_t H,
                  double *c, double *h, double *gates) {
#pragma omp parallel for schedule(static)
  for (int64_t b = 0; b < B; ++b) {
    for (int64_t j = 0; j < H; ++j) {
      const double *zr = z + b * 4 * H;
      double zi = zr[j], zf = zr[H + j], zg = zr[2 * H + j], zo = zr[3 * H + j];
      if (bias) { zi += bias[j]; zf += bias[H + j]; zg += bias[2 * H + j]; zo += bias[3 * H + j]; }
      double i = orc_sigmoid(zi), f = orc_sigmoid(zf), g = tanh(zg), o = orc_sigmoid(zo);
      double cn = f * c_prev[b * H + j] + i * g;
      c[b * H + j] = cn;
      h[b * H + j] = o * tanh(cn);
      if (gates) {
        double *gr = gates + b * 4 * H;
        gr[j] = i; gr[H + j] = f; gr[2 * H + j] = g; gr[3 * H + j] = o;
      }
    }
  }
}

/* Backward of the cell from retained OUTPUTS only (activated gates and c), the way the paper's
 * function-wise memory reduction describes for tanh-like operations:
 *   do = dh * tanh(c)            dc = dc_next + dh * o * (1 - tanh(c)^2)
 *   di = dc * g   dg = dc * i    df = dc * c_prev    dc_prev = dc * f
 *   dz_i = di i (1-i)   dz_f = df f (1-f)   dz_g = dg (1-g^2)   dz_o = do o (1-o)
 * dc_next may be NULL (zero). */
void orc_lstm_bwd(const double *gates, const double *c_prev, const double *c, const double *dh,
                  const double *dc_next, int64_t B, int64_t H, double *dz, double *dc_prev) {
#pragma omp parallel for schedule(static)
  for (int64_t b = 0; b < B; ++b) {
    for (int64_t j = 0; j < H; ++j) {
      const double *gr = gates + b * 4 * H;
      double i = gr[j], f = gr[H + j], g = gr[2 * H + j], o = gr[3 * H + j];
      double tc = tanh(c[b * H + j]);
      double dhv = dh[b * H + j];
      double d_o = dhv * tc;
      double dc = (dc_next ? dc_next[b * H + j] : 0.0) + dhv * o * (1.0 - tc * tc);
      double di = dc * g, dg = dc * i, df = dc * c_prev[b * H + j];
      dc_prev[b * H + j] = dc * f;
      double *dr = dz + b * 4 * H;
      dr[j] = di * i * (1.0 - i);
      dr[H + j] = df * f * (1.0 - f);
      dr[2 * H + j] = dg * (1.0 - g * g);
      dr[3 * H + j] = d_o * o * (1.0 - o);
    }
  }
}

/* Softmax cross-entropy, textbook form.  logits (N,C) contiguous, labels (N,).
 *   lse_n = m + log sum_c exp(z_nc - m), m = max_c z_nc ;  loss_n = lse_n - z[n, t_n]
 *   loss  = (1 / N_valid) sum over rows whose label != ignore_label
 * Rows with the ignored label have loss_n = 0.  N_valid = 0 gives loss 0.  A label outside [0, C)
 * counts as ignored (the boundary's rule for stray indices: never an offset, never an error).
 * Returns N_valid.  loss_rows, lse may be NULL. */
static int label_counts(int64_t t, int64_t ignore_label, int64_t C) {
  return t != ignore_label && t >= 0 && t < C;
}

int64_t orc_softmax_ce_fwd(const double *logits, const int64_t *labels, int64_t N, int64_t C,
                           int64_t ignore_label, double *loss_mean, double *loss_rows,
                           double *lse) {
  int64_t n_valid = 0;
  double total = 0.0;
  for (int64_t n = 0; n < N; ++n) {
    const double *z = logits + n * C;
    double m = -INFINITY;
    for (int64_t c = 0; c < C; ++c) if (z[c] > m) m = z[c];
    double s = 0.0;
    for (int64_t c = 0; c < C; ++c) s += exp(z[c] - m);
    double l = m + log(s);
    if (lse) lse[n] = l;
    double ln = 0.0;
    if (label_counts(labels[n], ignore_label, C)) { ln = l - z[labels[n]]; ++n_valid; total += ln; }
    if (loss_rows) loss_rows[n] = ln;
  }
  *loss_mean = n_valid > 0 ? total / (double)n_valid : 0.0;
  return n_valid;
}

/* Gradient of (upstream * mean loss) with respect to the logits:
 *   dz[n,c] = (upstream / N_valid) * (softmax(z)[n,c] - [c == t_n]); ignored rows get 0. */
void orc_softmax_ce_bwd(const double *logits, const int64_t *labels, int64_t N, int64_t C,
                        int64_t ignore_label, double upstream, double *dlogits) {
  int64_t n_valid = 0;
  for (int64_t n = 0; n < N; ++n) if (label_counts(labels[n], ignore_label, C)) ++n_valid;
  double g = n_valid > 0 ? upstream / (double)n_valid : 0.0;
#pragma omp parallel for schedule(static)
  for (int64_t n = 0; n < N; ++n) {
    const double *z = logits + n * C;
    double *d = dlogits + n * C;
    if (!label_counts(labels[n], ignore_label, C)) { for (int64_t c = 0; c < C; ++c) d[c] = 0.0; continue; }
    double m = -INFINITY;
    for (int64_t c = 0; c < C; ++c) if (z[c] > m) m = z[c];
    double s = 0.0;
    for (int64_t c = 0; c < C; ++c) s += exp(z[c] - m);
    for (int64_t c = 0; c < C; ++c) {
      double p = exp(z[c] - m) / s;
      d[c] = g * (p - (c == labels[n] ? 1.0 : 0.0));
    }
  }
}

/* The derivative of orc_softmax_ce_bwd (for a backward pass that is differentiated again): with
 * G[n,c] = s_n (p[n,c] - [c == t_n]), s_n = upstream / N_valid on valid rows, and u the gradient reaching G,
 *   dlogits[n,c] = s_n p[n,c] (u[n,c] - sum_k p[n,k] u[n,k]),
 *   *dupstream   = (1 / N_valid) sum over valid n, all c of u[n,c] (p[n,c] - [c == t_n]).
 * (d p_k / d z_c = p_k ([k == c] - p_c), the textbook softmax Jacobian.) */
void orc_softmax_ce_bwd2(const double *logits, const int64_t *labels, int64_t N, int64_t C,
                         int64_t ignore_label, double upstream, const double *u, double *dlogits,
                         double *dupstream) {
  int64_t n_valid = 0;
  for (int64_t n = 0; n < N; ++n) if (label_counts(labels[n], ignore_label, C)) ++n_valid;
  double s = n_valid > 0 ? upstream / (double)n_valid : 0.0;
  double du = 0.0;
  for (int64_t n = 0; n < N; ++n) {
    const double *z = logits + n * C, *un = u + n * C;
    double *d = dlogits + n * C;
    if (!label_counts(labels[n], ignore_label, C)) { for (int64_t c = 0; c < C; ++c) d[c] = 0.0; continue; }
    double m = -INFINITY;
    for (int64_t c = 0; c < C; ++c) if (z[c] > m) m = z[c];
    double sum = 0.0;
    for (int64_t c = 0; c < C; ++c) sum += exp(z[c] - m);
    double pu = 0.0;
    for (int64_t c = 0; c < C; ++c) pu += exp(z[c] - m) / sum * un[c];
    for (int64_t c = 0; c < C; ++c) d[c] = s * (exp(z[c] - m) / sum) * (un[c] - pu);
    du += pu - un[labels[n]];
  }
  if (dupstream) *dupstream = n_valid > 0 ? du / (double)n_valid : 0.0;
}

/* Plain stochastic gradient descent, p <- p - lr * g (no momentum, decay or clipping). */
void orc_sgd_update(double *p, const double *g, int64_t n, double lr) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) p[i] = p[i] - lr * g[i];
}

/* Embedding lookup out[n,:] = table[ids[n],:] and its gradient dtable[v,:] (+)= sum_{n: ids[n]=v} dout[n,:].
 * An id outside [0, V) selects no row: it gathers zeros and takes part in no sum. */
void orc_embed_fwd(const double *table, const int64_t *ids, int64_t N, int64_t D, int64_t V, double *out) {
#pragma omp parallel for schedule(static)
  for (int64_t n = 0; n < N; ++n)
    for (int64_t d = 0; d < D; ++d) out[n * D + d] = (ids[n] >= 0 && ids[n] < V) ? table[ids[n] * D + d] : 0.0;
}

void orc_embed_bwd(const int64_t *ids, const double *dout, int64_t N, int64_t D, int64_t V,
                   int accumulate, double *dtable) {
  if (!accumulate) for (int64_t i = 0; i < V * D; ++i) dtable[i] = 0.0;
  for (int64_t n = 0; n < N; ++n) {
    if (ids[n] < 0 || ids[n] >= V) continue;
    for (int64_t d = 0; d < D; ++d) dtable[ids[n] * D + d] += dout[n * D + d];
  }
}

/* Round each value to the nearest bfloat16 (8 significant bits, fp32 exponent range), ties to even,
 * written from the format's definition: scale so the unit in the last place is 1, round to the
 * nearest integer (the default rounding mode is ties-to-even), scale back. */
void orc_round_bf16(double *x, int64_t n) {
  for (int64_t i = 0; i < n; ++i) {
    double v = x[i];
    if (v == 0.0 || isnan(v) || isinf(v)) continue;
    int e;
    frexp(v, &e);         /* |v| = f * 2^e with f in [0.5, 1)  ->  exponent of leading bit is e-1 */
    int lead = e - 1;
    if (lead < -126) lead = -126; /* subnormal range keeps the quantum of the smallest normal */
    int q = lead - 7;             /* exponent of the last kept bit */
    double r = ldexp(nearbyint(ldexp(v, -q)), q);
    if (fabs(r) >= ldexp(1.0, 128)) r = v > 0 ? INFINITY : -INFINITY;
    x[i] = r;
  }
}

int orc_num_threads(void) {
  int n = 1;
#ifdef _OPENMP
#pragma omp parallel
  {
#pragma omp master
    n = omp_get_num_threads();
  }
#endif
  return n;
}
