/*
 * CPU oracle for the Spark-FFN sparse decode path and the Spark-attention decode path
 * (Spark Transformer, arXiv 2506.06644).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, double-precision statement of
 * what the path computes, written from the paper's definitions.  It shares no code, header,
 * table or helper with the HIP library, and the product never calls it: only tests/, the
 * smoke check and the benchmark's cpu_baseline leg may load it.
 *
 * Every sum below is a straight loop in double precision in the order the definition
 * states; there is no blocking, fusion or reordering.  OpenMP is used only across
 * independent outputs (rows / neurons / output columns), never inside a sum, so the value
 * of every output is the same for any thread count.
 *
 * Parity pins (tests/test_oracle_pins.py): quantile vs. textbook values and two library
 * routines; count ~ k on Gaussian rows; nesting with the sort-based top-m set by brute
 * force; zero/shift structure; affine and permutation equivariance; variational optimality;
 * GEMV / gathered-sum steps vs. float64 matmul; sparse == dense; the FLOP identities of
 * Eq.3/Eq.4.  Spark attention (Eq.7): the gated softmax lookup with library softmax /
 * logaddexp when every key is kept; the sort-based top-m set and the softmax restricted to it;
 * closed forms (zero gate keys and identical values give ln 2 times the value; identity values
 * expose p_i g_i; constant scores give 0); shift and permutation invariance; kept count ~ k.
 * The numeric values of y for the Gemma-shaped layers and caches have no printed example in
 * the paper: they are pinned only through the composition of these steps.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define REF_OK 0
#define REF_ERR_NULL 1
#define REF_ERR_SHAPE 2
#define REF_ERR_K 3

#define REF_FILL_ZERO 0
#define REF_FILL_NEG_INF 1

#define REF_GELU_ERF 0
#define REF_GELU_TANH 1

int spark_ref_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Standard normal CDF, Phi(z) = erfc(-z / sqrt 2) / 2. */
double spark_ref_normal_cdf(double z) { return 0.5 * erfc(-z / sqrt(2.0)); }

/*
 * Q(p): quantile of the standard Gaussian (Section 3, text after Eq.11).  The paper
 * leaves the evaluation method open, so the oracle solves Phi(z) = p directly: bisection on a
 * bracket that certainly contains the root, run until the bracket stops shrinking in
 * double precision.  For p > 1/2 the symmetric problem is solved so the tail keeps its
 * relative accuracy.
 */
double spark_ref_normal_quantile(double p) {
  if (!(p > 0.0) || !(p < 1.0)) {
    if (p == 0.0) return -INFINITY;
    if (p == 1.0) return INFINITY;
    return NAN;
  }
  if (p == 0.5) return 0.0;
  if (p > 0.5) return -spark_ref_normal_quantile(1.0 - p);
  double lo = -40.0, hi = 0.0; /* Phi(-40) underflows to 0 < p < 1/2 = Phi(0) */
  for (int it = 0; it < 400; ++it) {
    double mid = 0.5 * (lo + hi);
    if (mid <= lo || mid >= hi) break;
    if (spark_ref_normal_cdf(mid) < p)
      lo = mid;
    else
      hi = mid;
  }
  return 0.5 * (lo + hi);
}

/* GELU(x) = x * Phi(x) (exact form); the tanh form is the common approximation of it. */
double spark_ref_gelu(double x, int kind) {
  if (kind == REF_GELU_TANH) {
    const double c = sqrt(2.0 / acos(-1.0));
    return 0.5 * x * (1.0 + tanh(c * (x + 0.044715 * x * x * x)));
  }
  return 0.5 * x * (1.0 + erf(x / sqrt(2.0)));
}

/*
 * Statistical top-k of one vector (Eq.9, Eq.10, Eq.11).
 *   mean  = (1/d) sum x_i
 *   std   = sqrt( (1/(d-1)) sum (x_i - mean)^2 )
 *   theta = mean + std * Q(1 - k/d)
 *   y_i   = x_i - theta  if x_i > theta, else 0   (or -inf for the Top_k^(-inf) variant)
 * Active set = { i : x_i > theta } (strict, as counted in Theorem 1), ascending.
 * stats[4] = { mean, std, Q(1-k/d), theta }.  y, idx, count may be NULL.
 */
int spark_ref_stat_topk(const double* x, int64_t d, int64_t k, int fill, double* y,
                        double* stats, int32_t* idx, int64_t* count) {
  if (!x) return REF_ERR_NULL;
  if (d < 2) return REF_ERR_SHAPE;
  if (k < 1 || k > d - 1) return REF_ERR_K;
  double sum = 0.0;
  for (int64_t i = 0; i < d; ++i) sum += x[i];
  const double mean = sum / (double)d;
  double ss = 0.0;
  for (int64_t i = 0; i < d; ++i) {
    const double c = x[i] - mean;
    ss += c * c;
  }
  const double std = sqrt(ss / (double)(d - 1));
  const double z = spark_ref_normal_quantile(1.0 - (double)k / (double)d);
  const double theta = mean + std * z;
  int64_t m = 0;
  for (int64_t i = 0; i < d; ++i) {
    const int active = x[i] > theta;
    if (y) y[i] = active ? x[i] - theta : (fill == REF_FILL_NEG_INF ? -INFINITY : 0.0);
    if (active) {
      if (idx) idx[m] = (int32_t)i;
      ++m;
    }
  }
  if (stats) {
    stats[0] = mean;
    stats[1] = std;
    stats[2] = z;
    stats[3] = theta;
  }
  if (count) *count = m;
  return REF_OK;
}

/* Row-wise statistical top-k over x[rows][d] (the training / prefill shape). */
int spark_ref_stat_topk_rows(const double* x, int64_t rows, int64_t d, int64_t ldx, int64_t k,
                             int fill, double* y, int64_t ldy, double* theta, double* std,
                             int64_t* count, int32_t* idx, int64_t ldidx, int threads) {
  if (!x) return REF_ERR_NULL;
  if (rows < 0 || d < 2 || ldx < d || (y && ldy < d) || (idx && ldidx < d)) return REF_ERR_SHAPE;
  if (k < 1 || k > d - 1) return REF_ERR_K;
#ifdef _OPENMP
  if (threads <= 0) threads = omp_get_max_threads();
#endif
  (void)threads;
#pragma omp parallel for num_threads(threads) schedule(static)
  for (int64_t row = 0; row < rows; ++row) {
    double st[4];
    int64_t m = 0;
    spark_ref_stat_topk(x + row * ldx, d, k, fill, y ? y + row * ldy : NULL, st,
                        idx ? idx + row * ldidx : NULL, &m);
    if (theta) theta[row] = st[3];
    if (std) std[row] = st[1];
    if (count) count[row] = m;
  }
  return REF_OK;
}

/*
 * Huber loss (Section 3.2, Eq.13), entrywise: x^2 / 2 for |x| < delta, delta (|x| - delta / 2)
 * otherwise.
 */
double spark_ref_huber(double x, double delta) {
  const double ax = fabs(x);
  return ax < delta ? 0.5 * x * x : delta * (ax - 0.5 * delta);
}

/*
 * Huber statistical top-k of one vector (Section 3.2, Eq.14): y = Huber(StatTop_k(x); delta)
 * / delta, the continuously differentiable variant of Theorem 2.  delta = 0 is the limit
 * the paper uses in practice, y = StatTop_k(x) (StatTop_k(x) >= 0, so Huber / delta -> |.|
 * returns it unchanged).  stats as in spark_ref_stat_topk.
 */
int spark_ref_huber_stat_topk(const double* x, int64_t d, int64_t k, double delta, double* y,
                              double* stats) {
  if (!x || !y) return REF_ERR_NULL;
  if (!(delta >= 0.0)) return REF_ERR_SHAPE;
  const int rc = spark_ref_stat_topk(x, d, k, REF_FILL_ZERO, y, stats, NULL, NULL);
  if (rc != REF_OK) return rc;
  if (delta > 0.0)
    for (int64_t i = 0; i < d; ++i) y[i] = spark_ref_huber(y[i], delta) / delta;
  return REF_OK;
}

/*
 * Vector-Jacobian product of the Huber statistical top-k: gx_j = sum_i gy_i * dy_i / dx_j.
 * The operator is the composition used in the proof of Theorem 2 (Appendix A.2):
 *   theta(x) = mean + std * z,         z = Q(1 - k/d) a constant,
 *   y_i      = h(x_i, theta),          h = Huber(max(x - theta, 0); delta) / delta,
 * whose partial derivatives the proof lists (divided by delta here):
 *   dh/dx = -dh/dtheta = 1               for x > theta + delta,
 *                        (x - theta)/delta  for theta <= x <= theta + delta,
 *                        0               for x < theta
 * (for delta = 0: 1 for x > theta, 0 otherwise: soft thresholding, differentiable except where
 * an entry meets theta).  theta is a linear combination of the sample mean and the sample
 * standard deviation (Eq.9, Eq.11):
 *   d mean / dx_j = 1/d,   d std / dx_j = (x_j - mean) / ((d - 1) std).
 * Chain rule: gx_j = gy_j * dh/dx(x_j) - (sum_i gy_i * dh/dx(x_i)) * dtheta/dx_j.
 * A constant vector has std = 0: no entry exceeds theta, every dh/dx is 0 and gx = 0 (the
 * derivative of std does not exist there and is not needed).
 */
int spark_ref_huber_stat_topk_vjp(const double* x, const double* gy, int64_t d, int64_t k,
                                  double delta, double* gx) {
  if (!x || !gy || !gx) return REF_ERR_NULL;
  if (!(delta >= 0.0)) return REF_ERR_SHAPE;
  double st[4];
  const int rc = spark_ref_stat_topk(x, d, k, REF_FILL_ZERO, NULL, st, NULL, NULL);
  if (rc != REF_OK) return rc;
  const double mean = st[0], std = st[1], z = st[2], theta = st[3];
  double total = 0.0;
  for (int64_t i = 0; i < d; ++i) {
    const double a = x[i] - theta;
    double slope = 0.0;
    if (a > 0.0) slope = (delta > 0.0 && a < delta) ? a / delta : 1.0;
    gx[i] = gy[i] * slope;
    total += gy[i] * slope;
  }
  if (total != 0.0)
    for (int64_t j = 0; j < d; ++j) {
      const double dstd = std > 0.0 ? (x[j] - mean) / ((double)(d - 1) * std) : 0.0;
      gx[j] -= total * (1.0 / (double)d + z * dstd);
    }
  return REF_OK;
}

/* Row-wise forms over x[rows][d] (contiguous rows of length d). */
int spark_ref_huber_stat_topk_rows(const double* x, int64_t rows, int64_t d, int64_t k, double delta,
                                   double* y, double* theta, int threads) {
  if (!x || !y) return REF_ERR_NULL;
  if (rows < 0 || d < 2) return REF_ERR_SHAPE;
  if (k < 1 || k > d - 1) return REF_ERR_K;
  if (!(delta >= 0.0)) return REF_ERR_SHAPE;
#ifdef _OPENMP
  if (threads <= 0) threads = omp_get_max_threads();
#endif
  (void)threads;
#pragma omp parallel for num_threads(threads) schedule(static)
  for (int64_t row = 0; row < rows; ++row) {
    double st[4];
    spark_ref_huber_stat_topk(x + row * d, d, k, delta, y + row * d, st);
    if (theta) theta[row] = st[3];
  }
  return REF_OK;
}

int spark_ref_huber_stat_topk_vjp_rows(const double* x, const double* gy, int64_t rows, int64_t d,
                                       int64_t k, double delta, double* gx, int threads) {
  if (!x || !gy || !gx) return REF_ERR_NULL;
  if (rows < 0 || d < 2) return REF_ERR_SHAPE;
  if (k < 1 || k > d - 1) return REF_ERR_K;
  if (!(delta >= 0.0)) return REF_ERR_SHAPE;
#ifdef _OPENMP
  if (threads <= 0) threads = omp_get_max_threads();
#endif
  (void)threads;
#pragma omp parallel for num_threads(threads) schedule(static)
  for (int64_t row = 0; row < rows; ++row)
    spark_ref_huber_stat_topk_vjp(x + row * d, gy + row * d, d, k, delta, gx + row * d);
  return REF_OK;
}

/*
 * Exact top-k by sorting: indices of the k largest entries (ties: lower index first),
 * returned ascending by index.  Used to measure how far the statistical set is from the
 * sort-based one, and as the brute-force side of the nesting pin.
 */
typedef struct {
  double v;
  int32_t i;
} ref_pair;

static int ref_pair_desc(const void* a, const void* b) {
  const ref_pair* pa = (const ref_pair*)a;
  const ref_pair* pb = (const ref_pair*)b;
  if (pa->v > pb->v) return -1;
  if (pa->v < pb->v) return 1;
  return (pa->i > pb->i) - (pa->i < pb->i);
}

static int ref_i32_asc(const void* a, const void* b) {
  const int32_t ia = *(const int32_t*)a, ib = *(const int32_t*)b;
  return (ia > ib) - (ia < ib);
}

int spark_ref_exact_topk(const double* x, int64_t d, int64_t k, int32_t* idx) {
  if (!x || !idx) return REF_ERR_NULL;
  if (d < 1) return REF_ERR_SHAPE;
  if (k < 0 || k > d) return REF_ERR_K;
  ref_pair* p = (ref_pair*)malloc((size_t)d * sizeof(ref_pair));
  if (!p) return REF_ERR_SHAPE;
  for (int64_t i = 0; i < d; ++i) {
    p[i].v = x[i];
    p[i].i = (int32_t)i;
  }
  qsort(p, (size_t)d, sizeof(ref_pair), ref_pair_desc);
  for (int64_t i = 0; i < k; ++i) idx[i] = p[i].i;
  qsort(idx, (size_t)k, sizeof(int32_t), ref_i32_asc);
  free(p);
  return REF_OK;
}

int spark_ref_exact_topk_rows(const double* x, int64_t rows, int64_t d, int64_t ldx, int64_t k,
                              int32_t* idx, int threads) {
  if (!x || !idx) return REF_ERR_NULL;
#ifdef _OPENMP
  if (threads <= 0) threads = omp_get_max_threads();
#endif
  (void)threads;
  int rc = REF_OK;
#pragma omp parallel for num_threads(threads) schedule(static) reduction(max : rc)
  for (int64_t row = 0; row < rows; ++row) {
    int e = spark_ref_exact_topk(x + row * ldx, d, k, idx + row * k);
    if (e > rc) rc = e;
  }
  return rc;
}

/*
 * Value of an 8-bit floating-point code in the OCP "E4M3" format (1 sign, 4 exponent bits with
 * bias 7, 3 mantissa bits; no infinities; exponent 15 with mantissa 7 is NaN; exponent 0 holds
 * the subnormals m / 8 * 2^-6; largest finite value 448).  This is the storage format of the
 * low-precision weight rows (the quantisation synergy of Appendix D.4): a stored row is its
 * codes and one fp32 scale, weight = scale * value(code).
 */
double spark_ref_fp8_e4m3_value(unsigned code) {
  const unsigned sign = (code >> 7) & 1u, e = (code >> 3) & 15u, m = code & 7u;
  double v;
  if (e == 15u && m == 7u) return NAN;
  if (e == 0u) v = ldexp((double)m / 8.0, -6);
  else v = ldexp(1.0 + (double)m / 8.0, (int)e - 7);
  return sign ? -v : v;
}

/* weight[row][c] = scale[row] * value(code[row][c]) for rows x cols codes, as float (exact when
 * the scale has at most 20 significant bits; the synthetic inputs keep to 8). */
int spark_ref_fp8_dequantize_rows(const uint8_t* codes, const float* scales, int64_t rows, int64_t cols,
                                  float* out) {
  if (!codes || !scales || !out) return REF_ERR_NULL;
  if (rows < 0 || cols < 0) return REF_ERR_SHAPE;
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t c = 0; c < cols; ++c)
      out[r * cols + c] = (float)((double)scales[r] * spark_ref_fp8_e4m3_value(codes[r * cols + c]));
  return REF_OK;
}

/* The same for signed 8-bit integer codes (two's complement): weight = scale * code. */
int spark_ref_int8_dequantize_rows(const int8_t* codes, const float* scales, int64_t rows, int64_t cols,
                                   float* out) {
  if (!codes || !scales || !out) return REF_ERR_NULL;
  if (rows < 0 || cols < 0) return REF_ERR_SHAPE;
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t c = 0; c < cols; ++c) out[r * cols + c] = (float)((double)scales[r] * (double)codes[r * cols + c]);
  return REF_OK;
}

/*
 * One Spark-FFN layer for one token (Eq.2), weights neuron-major (row j = column j of the
 * paper's K1 / K2 / V):
 *   s_j = sum_{i<r} K1n[j][i] * q[i]                          predictor, all j
 *   a   = StatTop_k(s)                                        Eq.10
 *   g_j = sum_{i<d_model-r} K2n[j][i] * q[r+i]
 *   u_j = GELU(a_j) * g_j                                     sigma = GELU on the shifted value
 *   y_c = sum_j u_j * Vn[j][c]
 * skip_inactive = 0: the dense definition (every j in every sum).
 * skip_inactive = 1: g and the y-sum run over the active set only; the skipped terms are
 *                    exact zeros (GELU(0) = 0), so both give the same y.
 * Weights and q arrive as float (the exact widening of their bf16 / fp32 storage).
 * Outputs (any may be NULL): y[d_model], s[d_ff], a[d_ff], u[d_ff], stats[4], idx[d_ff],
 * count, macs[3] = multiply-adds spent on K1, K2, V.
 */
int spark_ref_spark_ffn(const float* k1n, const float* k2n, const float* vn, const float* q,
                        int64_t d_model, int64_t d_ff, int64_t r, int64_t k, int gelu_kind,
                        int skip_inactive, double* y, double* s_out, double* a_out,
                        double* u_out, double* stats, int32_t* idx_out, int64_t* count_out,
                        int64_t* macs, int threads) {
  if (!k1n || !k2n || !vn || !q) return REF_ERR_NULL;
  if (d_ff < 2 || d_model < 2 || r < 1 || r > d_model - 1) return REF_ERR_SHAPE;
  if (k < 1 || k > d_ff - 1) return REF_ERR_K;
#ifdef _OPENMP
  if (threads <= 0) threads = omp_get_max_threads();
#endif
  (void)threads;
  const int64_t r2 = d_model - r;
  double* s = (double*)malloc((size_t)d_ff * sizeof(double));
  double* a = (double*)malloc((size_t)d_ff * sizeof(double));
  double* u = (double*)malloc((size_t)d_ff * sizeof(double));
  int32_t* idx = (int32_t*)malloc((size_t)d_ff * sizeof(int32_t));
  if (!s || !a || !u || !idx) {
    free(s); free(a); free(u); free(idx);
    return REF_ERR_SHAPE;
  }
  int64_t mac1 = 0, mac2 = 0, mac3 = 0;

#pragma omp parallel for num_threads(threads) schedule(static)
  for (int64_t j = 0; j < d_ff; ++j) {
    double acc = 0.0;
    for (int64_t i = 0; i < r; ++i) acc += (double)k1n[j * r + i] * (double)q[i];
    s[j] = acc;
  }
  mac1 = d_ff * r;

  double st[4];
  int64_t m = 0;
  int rc = spark_ref_stat_topk(s, d_ff, k, REF_FILL_ZERO, a, st, idx, &m);
  if (rc != REF_OK) {
    free(s); free(a); free(u); free(idx);
    return rc;
  }

  if (skip_inactive) {
    for (int64_t j = 0; j < d_ff; ++j) u[j] = 0.0;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int64_t t = 0; t < m; ++t) {
      const int64_t j = idx[t];
      double g = 0.0;
      for (int64_t i = 0; i < r2; ++i) g += (double)k2n[j * r2 + i] * (double)q[r + i];
      u[j] = spark_ref_gelu(a[j], gelu_kind) * g;
    }
    mac2 = m * r2;
  } else {
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int64_t j = 0; j < d_ff; ++j) {
      double g = 0.0;
      for (int64_t i = 0; i < r2; ++i) g += (double)k2n[j * r2 + i] * (double)q[r + i];
      u[j] = spark_ref_gelu(a[j], gelu_kind) * g;
    }
    mac2 = d_ff * r2;
  }

  if (y) {
    if (skip_inactive) {
#pragma omp parallel for num_threads(threads) schedule(static)
      for (int64_t c = 0; c < d_model; ++c) {
        double acc = 0.0;
        for (int64_t t = 0; t < m; ++t) {
          const int64_t j = idx[t];
          acc += u[j] * (double)vn[j * d_model + c];
        }
        y[c] = acc;
      }
      mac3 = m * d_model;
    } else {
#pragma omp parallel for num_threads(threads) schedule(static)
      for (int64_t c = 0; c < d_model; ++c) {
        double acc = 0.0;
        for (int64_t j = 0; j < d_ff; ++j) acc += u[j] * (double)vn[j * d_model + c];
        y[c] = acc;
      }
      mac3 = d_ff * d_model;
    }
  }

  if (s_out) memcpy(s_out, s, (size_t)d_ff * sizeof(double));
  if (a_out) memcpy(a_out, a, (size_t)d_ff * sizeof(double));
  if (u_out) memcpy(u_out, u, (size_t)d_ff * sizeof(double));
  if (idx_out) memcpy(idx_out, idx, (size_t)m * sizeof(int32_t));
  if (stats) memcpy(stats, st, sizeof(st));
  if (count_out) *count_out = m;
  if (macs) {
    macs[0] = mac1;
    macs[1] = mac2;
    macs[2] = mac3;
  }
  free(s); free(a); free(u); free(idx);
  return REF_OK;
}

/* Entrywise softplus, log(1 + exp(x)), evaluated without overflow. */
double spark_ref_softplus(double x) { return x > 0.0 ? x + log1p(exp(-x)) : log1p(exp(x)); }

/*
 * One head of Spark attention for one query (Eq.7, with Top_k^(-inf) as described after
 * Eq.11).  Caches are token-major ("row format"): k1c[n_ctx][r] holds the first r entries of
 * every key, k2c[n_ctx][d_attn - r] the rest, vc[n_ctx][d_attn] the values.
 *
 *   s_i = sum_{t<r} k1c[i][t] * q[t]                              predictor scores
 *   a   = StatTop_k^(-inf)(s):  a_i = s_i - theta if s_i > theta, else -inf
 *   p   = softmax(a)            (entries at -inf get weight 0)
 *   g_i = softplus( sum_{t<d_attn-r} k2c[i][t] * q[r+t] )
 *   y_c = sum_i p_i * g_i * vc[i][c]
 *
 * Readings where the paper is silent: when n_ctx <= k every key is kept (the FLOP count uses
 * min{k, n_ctx}), i.e. theta = -inf and a = s; when no score exceeds theta (all scores
 * equal) the softmax has nothing to normalise and y = 0.  No 1/sqrt(d) factor is applied:
 * Eq.5 and Eq.7 carry none (a caller folds it into q).
 * Outputs (any may be NULL): y[d_attn], s[n_ctx], p[n_ctx], g[n_ctx] (0 where p_i = 0 and
 * skip_inactive is set), stats[4] = {mean, std, Q, theta}, idx[count], count.
 */
int spark_ref_spark_attention(const float* k1c, const float* k2c, const float* vc, const float* q,
                              int64_t n_ctx, int64_t d_attn, int64_t r, int64_t k,
                              int skip_inactive, double* y, double* s_out, double* p_out,
                              double* g_out, double* stats, int32_t* idx_out, int64_t* count_out) {
  if (!k1c || !k2c || !vc || !q) return REF_ERR_NULL;
  if (n_ctx < 1 || d_attn < 2 || r < 1 || r > d_attn - 1) return REF_ERR_SHAPE;
  if (k < 1) return REF_ERR_K;
  const int64_t r2 = d_attn - r;
  double* s = (double*)malloc((size_t)n_ctx * sizeof(double));
  double* a = (double*)malloc((size_t)n_ctx * sizeof(double));
  double* p = (double*)malloc((size_t)n_ctx * sizeof(double));
  double* g = (double*)malloc((size_t)n_ctx * sizeof(double));
  int32_t* idx = (int32_t*)malloc((size_t)n_ctx * sizeof(int32_t));
  if (!s || !a || !p || !g || !idx) {
    free(s); free(a); free(p); free(g); free(idx);
    return REF_ERR_SHAPE;
  }
  for (int64_t i = 0; i < n_ctx; ++i) {
    double acc = 0.0;
    for (int64_t t = 0; t < r; ++t) acc += (double)k1c[i * r + t] * (double)q[t];
    s[i] = acc;
  }
  double st[4] = {0.0, 0.0, 0.0, -INFINITY};
  int64_t m = 0;
  if (n_ctx <= k) {
    for (int64_t i = 0; i < n_ctx; ++i) {
      a[i] = s[i];
      idx[i] = (int32_t)i;
    }
    m = n_ctx;
  } else {
    const int rc = spark_ref_stat_topk(s, n_ctx, k, REF_FILL_NEG_INF, a, st, idx, &m);
    if (rc != REF_OK) {
      free(s); free(a); free(p); free(g); free(idx);
      return rc;
    }
  }
  /* softmax over the kept entries, shifted by their maximum */
  double amax = -INFINITY;
  for (int64_t i = 0; i < n_ctx; ++i)
    if (a[i] > amax) amax = a[i];
  double den = 0.0;
  for (int64_t i = 0; i < n_ctx; ++i) {
    p[i] = a[i] == -INFINITY ? 0.0 : exp(a[i] - amax);
    den += p[i];
  }
  for (int64_t i = 0; i < n_ctx; ++i) p[i] = den > 0.0 ? p[i] / den : 0.0;
  for (int64_t i = 0; i < n_ctx; ++i) {
    if (skip_inactive && p[i] == 0.0) {
      g[i] = 0.0;
      continue;
    }
    double acc = 0.0;
    for (int64_t t = 0; t < r2; ++t) acc += (double)k2c[i * r2 + t] * (double)q[r + t];
    g[i] = spark_ref_softplus(acc);
  }
  if (y) {
    for (int64_t c = 0; c < d_attn; ++c) {
      double acc = 0.0;
      for (int64_t i = 0; i < n_ctx; ++i) {
        if (skip_inactive && p[i] == 0.0) continue;
        acc += p[i] * g[i] * (double)vc[i * d_attn + c];
      }
      y[c] = acc;
    }
  }
  if (s_out) memcpy(s_out, s, (size_t)n_ctx * sizeof(double));
  if (p_out) memcpy(p_out, p, (size_t)n_ctx * sizeof(double));
  if (g_out) memcpy(g_out, g, (size_t)n_ctx * sizeof(double));
  if (idx_out) memcpy(idx_out, idx, (size_t)m * sizeof(int32_t));
  if (stats) memcpy(stats, st, sizeof(st));
  if (count_out) *count_out = m;
  free(s); free(a); free(p); free(g); free(idx);
  return REF_OK;
}

/*
 * Eq.7 with the kept set handed in instead of derived: the softmax runs over exactly the keys
 * kept[0..m) (every other key has weight 0, as after Top_k^(-inf)), gated by softplus and
 * applied to the values,
 *   y_c = sum_{i in kept} softmax_kept(s)_i * softplus(k2c[i] . q[r:]) * vc[i][c],
 *   s_i = k1c[i] . q[:r].
 * The softmax is invariant to the shift by theta, so the scores themselves are used.  It says
 * what Eq.7 yields for a kept set that differs from the oracle's own by keys sitting at the
 * threshold.  m = 0 gives y = 0.
 */
int spark_ref_spark_attention_on_set(const float* k1c, const float* k2c, const float* vc, const float* q,
                                     int64_t n_ctx, int64_t d_attn, int64_t r, const int32_t* kept,
                                     int64_t m, double* y) {
  if (!k1c || !k2c || !vc || !q || !y || (m > 0 && !kept)) return REF_ERR_NULL;
  if (n_ctx < 1 || d_attn < 2 || r < 1 || r > d_attn - 1 || m < 0 || m > n_ctx) return REF_ERR_SHAPE;
  const int64_t r2 = d_attn - r;
  for (int64_t c = 0; c < d_attn; ++c) y[c] = 0.0;
  if (m == 0) return REF_OK;
  double* s = (double*)malloc((size_t)m * sizeof(double));
  double* w = (double*)malloc((size_t)m * sizeof(double));
  if (!s || !w) {
    free(s); free(w);
    return REF_ERR_SHAPE;
  }
  double smax = -INFINITY;
  for (int64_t t = 0; t < m; ++t) {
    const int64_t i = kept[t];
    if (i < 0 || i >= n_ctx) {
      free(s); free(w);
      return REF_ERR_SHAPE;
    }
    double acc = 0.0;
    for (int64_t e = 0; e < r; ++e) acc += (double)k1c[i * r + e] * (double)q[e];
    s[t] = acc;
    if (acc > smax) smax = acc;
  }
  double den = 0.0;
  for (int64_t t = 0; t < m; ++t) {
    w[t] = exp(s[t] - smax);
    den += w[t];
  }
  for (int64_t t = 0; t < m; ++t) {
    const int64_t i = kept[t];
    double acc = 0.0;
    for (int64_t e = 0; e < r2; ++e) acc += (double)k2c[i * r2 + e] * (double)q[r + e];
    w[t] = w[t] / den * spark_ref_softplus(acc);
  }
  for (int64_t c = 0; c < d_attn; ++c) {
    double acc = 0.0;
    for (int64_t t = 0; t < m; ++t) acc += w[t] * (double)vc[(int64_t)kept[t] * d_attn + c];
    y[c] = acc;
  }
  free(s); free(w);
  return REF_OK;
}
