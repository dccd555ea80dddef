/*
 * LAQ oracle, model gradients -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Local gradients grad f_m(theta) of the losses in the supplement
 * ("Simulation details"): regularised multinomial logistic regression and a
 * fully connected ReLU network with softmax cross-entropy, plus the binary
 * logistic loss used by the smallest synthetic workload.  The global loss is
 * the mean over all N samples, so worker m returns
 *     g_m = (1/N) sum_{n in m} grad CE_n(theta) + (N_m/N) lambda theta
 * (each per-sample loss carries (lambda/2)||theta||^2).  One sample at a time,
 * every sum in double, one rounding to float at the end.
 */
#include "laq_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

void laq_oracle_grad_binlog(const float* theta, const float* X,
                            const int32_t* y, int64_t N_m, int64_t F,
                            int64_t ldx, int64_t N_total, float lambda,
                            float* g, double* loss_sum) {
  double* acc = (double*)calloc((size_t)F, sizeof(double));
  double loss = 0.0;
  for (int64_t n = 0; n < N_m; ++n) {
    const float* x = X + n * ldx;
    double z = 0.0;
    for (int64_t f = 0; f < F; ++f) z += (double)theta[f] * (double)x[f];
    double yy = (double)y[n];
    double marg = yy * z;
    /* l = log(1+exp(-marg));  dl/dz = -y / (1+exp(marg)) */
    loss += (marg > 0) ? log1p(exp(-marg)) : -marg + log1p(exp(marg));
    double coef = -yy / (1.0 + exp(marg));
    for (int64_t f = 0; f < F; ++f) acc[f] += coef * (double)x[f];
  }
  double invN = 1.0 / (double)N_total;
  double reg = ((double)N_m / (double)N_total) * (double)lambda;
  for (int64_t f = 0; f < F; ++f)
    g[f] = (float)(acc[f] * invN + reg * (double)theta[f]);
  if (loss_sum) *loss_sum = loss;
  free(acc);
}

void laq_oracle_grad_softmax(const float* theta, const float* X,
                             const int32_t* y, int64_t N_m, int64_t F,
                             int64_t ldx, int32_t C, int64_t N_total,
                             float lambda, float* g, double* loss_sum) {
  double* acc = (double*)calloc((size_t)C * (size_t)F, sizeof(double));
  double* z = (double*)malloc((size_t)C * sizeof(double));
  double loss = 0.0;
  for (int64_t n = 0; n < N_m; ++n) {
    const float* x = X + n * ldx;
    double zmax = -INFINITY;
    for (int32_t c = 0; c < C; ++c) {
      double s = 0.0;
      for (int64_t f = 0; f < F; ++f)
        s += (double)theta[(int64_t)c * F + f] * (double)x[f];
      z[c] = s;
      if (s > zmax) zmax = s;
    }
    double den = 0.0;
    for (int32_t c = 0; c < C; ++c) den += exp(z[c] - zmax);
    loss += -(z[y[n]] - zmax - log(den));
    for (int32_t c = 0; c < C; ++c) {
      double r = exp(z[c] - zmax) / den - (c == y[n] ? 1.0 : 0.0);
      for (int64_t f = 0; f < F; ++f)
        acc[(int64_t)c * F + f] += r * (double)x[f];
    }
  }
  double invN = 1.0 / (double)N_total;
  double reg = ((double)N_m / (double)N_total) * (double)lambda;
  for (int64_t i = 0; i < (int64_t)C * F; ++i)
    g[i] = (float)(acc[i] * invN + reg * (double)theta[i]);
  if (loss_sum) *loss_sum = loss;
  free(acc);
  free(z);
}

int64_t laq_oracle_mlp_params(const int32_t* dims, int32_t n_dims) {
  int64_t p = 0;
  for (int32_t l = 1; l < n_dims; ++l)
    p += (int64_t)dims[l - 1] * dims[l] + dims[l];
  return p;
}

void laq_oracle_grad_mlp(const float* theta, const float* X, const int32_t* y,
                         int64_t N_m, int64_t ldx, const int32_t* dims,
                         int32_t n_dims, int64_t N_total, float lambda,
                         float* g, double* loss_sum) {
  const int32_t nl = n_dims - 1;            /* number of weight layers */
  const int64_t p = laq_oracle_mlp_params(dims, n_dims);
  int64_t* offW = (int64_t*)malloc((size_t)nl * sizeof(int64_t));
  int64_t* offB = (int64_t*)malloc((size_t)nl * sizeof(int64_t));
  int64_t off = 0;
  int32_t wmax = 0;
  for (int32_t l = 0; l < nl; ++l) {
    offW[l] = off; off += (int64_t)dims[l] * dims[l + 1];
    offB[l] = off; off += dims[l + 1];
  }
  for (int32_t l = 0; l < n_dims; ++l) if (dims[l] > wmax) wmax = dims[l];

  double loss = 0.0;
  double* acc_all = (double*)calloc((size_t)p, sizeof(double));
  /* per-thread partial sums, combined afterwards in thread order so that the
   * result does not depend on which thread finishes first */
  int n_thr = 1;
#ifdef _OPENMP
  n_thr = omp_in_parallel() ? 1 : omp_get_max_threads();
#endif
  double** part = (double**)calloc((size_t)n_thr, sizeof(double*));
  double* part_loss = (double*)calloc((size_t)n_thr, sizeof(double));

#pragma omp parallel num_threads(n_thr)
  {
    int tid = 0;
#ifdef _OPENMP
    tid = omp_get_thread_num();
#endif
    double* acc = (double*)calloc((size_t)p, sizeof(double));
    part[tid] = acc;
    /* a[l] = activations entering layer l (a[0] = x), z[l] = pre-activations */
    double** a = (double**)malloc((size_t)(nl + 1) * sizeof(double*));
    double** z = (double**)malloc((size_t)nl * sizeof(double*));
    for (int32_t l = 0; l <= nl; ++l) a[l] = (double*)malloc((size_t)wmax * sizeof(double));
    for (int32_t l = 0; l < nl; ++l) z[l] = (double*)malloc((size_t)wmax * sizeof(double));
    double* dz = (double*)malloc((size_t)wmax * sizeof(double));
    double* da = (double*)malloc((size_t)wmax * sizeof(double));
    double my_loss = 0.0;

#pragma omp for schedule(static)
    for (int64_t n = 0; n < N_m; ++n) {
      const float* x = X + n * ldx;
      for (int32_t i = 0; i < dims[0]; ++i) a[0][i] = (double)x[i];
      /* forward */
      for (int32_t l = 0; l < nl; ++l) {
        const int32_t in = dims[l], out = dims[l + 1];
        const float* W = theta + offW[l];
        const float* B = theta + offB[l];
        for (int32_t j = 0; j < out; ++j) z[l][j] = (double)B[j];
        for (int32_t i = 0; i < in; ++i) {
          double ai = a[l][i];
          if (ai == 0.0) continue;          /* adds exact zeros: no effect */
          for (int32_t j = 0; j < out; ++j)
            z[l][j] += ai * (double)W[(int64_t)i * out + j];
        }
        if (l + 1 < nl)
          for (int32_t j = 0; j < out; ++j) a[l + 1][j] = z[l][j] > 0.0 ? z[l][j] : 0.0;
      }
      /* softmax cross-entropy on z[nl-1] */
      const int32_t C = dims[nl];
      double zmax = -INFINITY, den = 0.0;
      for (int32_t c = 0; c < C; ++c) if (z[nl - 1][c] > zmax) zmax = z[nl - 1][c];
      for (int32_t c = 0; c < C; ++c) den += exp(z[nl - 1][c] - zmax);
      my_loss += -(z[nl - 1][y[n]] - zmax - log(den));
      for (int32_t c = 0; c < C; ++c)
        dz[c] = exp(z[nl - 1][c] - zmax) / den - (c == y[n] ? 1.0 : 0.0);
      /* backward */
      for (int32_t l = nl - 1; l >= 0; --l) {
        const int32_t in = dims[l], out = dims[l + 1];
        const float* W = theta + offW[l];
        for (int32_t j = 0; j < out; ++j) acc[offB[l] + j] += dz[j];
        for (int32_t i = 0; i < in; ++i) {
          double ai = a[l][i];
          double s = 0.0;
          for (int32_t j = 0; j < out; ++j) {
            acc[offW[l] + (int64_t)i * out + j] += ai * dz[j];
            s += (double)W[(int64_t)i * out + j] * dz[j];
          }
          da[i] = s;
        }
        if (l > 0)
          for (int32_t i = 0; i < in; ++i) dz[i] = z[l - 1][i] > 0.0 ? da[i] : 0.0;
      }
    }

    part_loss[tid] = my_loss;
    for (int32_t l = 0; l <= nl; ++l) free(a[l]);
    for (int32_t l = 0; l < nl; ++l) free(z[l]);
    free(a); free(z); free(dz); free(da);
  }
  for (int th = 0; th < n_thr; ++th) {
    if (!part[th]) continue;
    for (int64_t i = 0; i < p; ++i) acc_all[i] += part[th][i];
    loss += part_loss[th];
    free(part[th]);
  }
  free(part); free(part_loss);

  double invN = 1.0 / (double)N_total;
  double reg = ((double)N_m / (double)N_total) * (double)lambda;
  for (int64_t i = 0; i < p; ++i)
    g[i] = (float)(acc_all[i] * invN + reg * (double)theta[i]);
  if (loss_sum) *loss_sum = loss;
  free(acc_all); free(offW); free(offB);
}

/* All M workers' gradients; X is [M][N_m][ldx], y is [M][N_m], G is [M][p].
 * kind: 1 binary logistic (dims[0]=F), 2 multinomial logistic
 * (dims = {F, C}), 3 ReLU network (dims = layer widths).  Returns the global
 * loss (1/N) sum_m f_m(theta) including the regulariser. */
double laq_oracle_grads_all(int32_t kind, const float* theta, const float* X,
                            const int32_t* y, int32_t M, int64_t N_m,
                            int64_t ldx, const int32_t* dims, int32_t n_dims,
                            float lambda, float* G) {
  const int64_t N = (int64_t)M * N_m;
  int64_t p;
  if (kind == 1) p = dims[0];
  else if (kind == 2) p = (int64_t)dims[0] * dims[1];
  else p = laq_oracle_mlp_params(dims, n_dims);
  double* loss = (double*)calloc((size_t)M, sizeof(double));
  if (kind == 3) {
    for (int32_t m = 0; m < M; ++m)
      laq_oracle_grad_mlp(theta, X + (int64_t)m * N_m * ldx, y + (int64_t)m * N_m,
                          N_m, ldx, dims, n_dims, N, lambda, G + (int64_t)m * p,
                          &loss[m]);
  } else {
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t m = 0; m < M; ++m) {
      const float* Xm = X + (int64_t)m * N_m * ldx;
      const int32_t* ym = y + (int64_t)m * N_m;
      if (kind == 1)
        laq_oracle_grad_binlog(theta, Xm, ym, N_m, dims[0], ldx, N, lambda,
                               G + (int64_t)m * p, &loss[m]);
      else
        laq_oracle_grad_softmax(theta, Xm, ym, N_m, dims[0], ldx, dims[1], N,
                                lambda, G + (int64_t)m * p, &loss[m]);
    }
  }
  double tot = 0.0, th2 = 0.0;
  for (int32_t m = 0; m < M; ++m) tot += loss[m];
  for (int64_t i = 0; i < p; ++i) th2 += (double)theta[i] * (double)theta[i];
  free(loss);
  return tot / (double)N + 0.5 * (double)lambda * th2;
}

/* Minibatch gradients for the stochastic variant (Sec. 4, "Stochastic
 * gradient-based tests": SLAQ is LAQ run on minibatch gradients).  Worker m
 * draws B of its N_m samples, idx[m][0..B) (indices into its own shard, drawn
 * by the caller), and returns the gradient of the loss its minibatch defines
 * under the same mean convention:
 *     g_m = (1/(M B)) sum_{j<B} grad CE_{idx[m][j]}(theta) + (1/M) lambda theta,
 * an unbiased estimate of the full g_m = (1/N) sum_n grad CE_n + (N_m/N) lambda theta
 * when the shards have equal size (N = M N_m).  Written as: copy the B drawn
 * rows out, then take the full gradient of that B-sample shard with N = M B. */
void laq_oracle_grads_minibatch(int32_t kind, const float* theta, const float* X,
                                const int32_t* y, int32_t M, int64_t N_m,
                                int64_t ldx, const int32_t* dims, int32_t n_dims,
                                float lambda, const int32_t* idx, int64_t B,
                                float* G) {
  float* Xb = (float*)malloc((size_t)M * (size_t)B * (size_t)ldx * sizeof(float));
  int32_t* yb = (int32_t*)malloc((size_t)M * (size_t)B * sizeof(int32_t));
  for (int32_t m = 0; m < M; ++m) {
    for (int64_t j = 0; j < B; ++j) {
      const int64_t n = idx[(int64_t)m * B + j];
      memcpy(Xb + ((int64_t)m * B + j) * ldx, X + ((int64_t)m * N_m + n) * ldx,
             (size_t)ldx * sizeof(float));
      yb[(int64_t)m * B + j] = y[(int64_t)m * N_m + n];
    }
  }
  (void)laq_oracle_grads_all(kind, theta, Xb, yb, M, B, ldx, dims, n_dims, lambda, G);
  free(Xb);
  free(yb);
}
