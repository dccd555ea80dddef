/*
 * LAQ oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE (see laq_oracle.h).
 *
 * Quantizer (Sec. 2.1, eqs. 5-6), skip rule (Sec. 2.2, eqs. 7a-7b), server
 * update (eq. 4) and the loop body of Algorithm 2, written step by step in
 * the paper's order and notation.  No blocking, no fusion.
 *
 * Finite-precision reading (the paper states eq. 5 over the reals): every
 * operation below that is marked fp32 is ONE IEEE-754 binary32 operation,
 * round-to-nearest-even, never fused.  The file must be compiled with
 * -ffp-contract=off.
 */
#include "laq_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

static int32_t ceil_log2_i64(int64_t n) {
  int32_t c = 0;
  while (((int64_t)1 << c) < n) ++c;
  return c;
}

/* Order-free squared error.  In fp32, eps_i = g_i - fl(h_i + delta_i) obeys
 * |eps_i| <= 2 tau R (1 + small): the rounding of h_i + delta_i can add up to
 * another |d_i - delta_i| because g_i itself is a representable candidate.
 * With 2^(x-1) <= step < 2^x each eps_i is rounded to the grid 2^(x-K) and the
 * squares are summed as integers; K is the largest exponent (capped at 20)
 * for which p * (1.04 * 2^K)^2 < 2^64. */
int32_t laq_oracle_eps_K(int64_t p) {
  int32_t K = (63 - ceil_log2_i64(p)) / 2;
  return K < 20 ? K : 20;
}

int64_t laq_oracle_code_words(int64_t p, int32_t b) {
  if (b == LAQ_ORACLE_B_EXACT) return p;
  return (p * (int64_t)b + 31) / 32;
}

int laq_oracle_quantize(const float* g, const float* h, int64_t p, int32_t b,
                        float* R_out, uint32_t* q, float* delta, float* h_new,
                        int64_t* Sq_out, double* E2_out, double* lhs_out) {
  /* radius R = || g - h ||_inf  (Sec. 2.1) */
  float R = 0.0f;
  int nonfinite = 0;
  for (int64_t i = 0; i < p; ++i) {
    float d = g[i] - h[i];                 /* fp32 */
    float a = fabsf(d);
    if (a != a) nonfinite = 1;
    if (a > R) R = a;
  }
  if (R_out) *R_out = nonfinite ? NAN : R;
  float two_R = 2.0f * R;                  /* fp32, exact unless overflow */
  if (nonfinite || !isfinite(R) || !isfinite(two_R)) return LAQ_ORACLE_ENONFINITE;

  if (b == LAQ_ORACLE_B_EXACT) {
    /* identity quantizer: Q_m(theta^k) = g, eps = 0 */
    double s2 = 0.0;
    for (int64_t i = 0; i < p; ++i) {
      float d = g[i] - h[i];               /* fp32 */
      if (delta) delta[i] = d;
      if (h_new) h_new[i] = g[i];
      if (q) memcpy(&q[i], &g[i], 4);
      s2 += (double)d * (double)d;
    }
    if (Sq_out) *Sq_out = 0;
    if (E2_out) *E2_out = 0.0;
    if (lhs_out) *lhs_out = s2;
    return LAQ_ORACLE_OK;
  }

  const int64_t L = ((int64_t)1 << b) - 1;  /* tau = 1/L */
  const float Lf = (float)L;
  const float s = Lf / two_R;               /* fp32: 1/(2 tau R) */
  const float step = two_R / Lf;            /* fp32: 2 tau R     */

  if (R == 0.0f || !isfinite(s)) {
    /* zero (or unrepresentably small) innovation: eq. 5 is 0/0 */
    for (int64_t i = 0; i < p; ++i) {
      if (q) q[i] = 0;
      if (delta) delta[i] = 0.0f;
      if (h_new) h_new[i] = h[i];
    }
    if (Sq_out) *Sq_out = 0;
    if (E2_out) *E2_out = 0.0;
    if (lhs_out) *lhs_out = 0.0;
    return LAQ_ORACLE_OK;
  }

  int x;
  (void)frexpf(step, &x);                   /* 2^(x-1) <= step < 2^x */
  const int32_t K = laq_oracle_eps_K(p);

  int64_t Sq = 0;
  uint64_t N = 0;
  for (int64_t i = 0; i < p; ++i) {
    /* eq. 5: q_i = floor( (d_i + R) / (2 tau R) + 1/2 ) */
    float d = g[i] - h[i];                  /* fp32 */
    float u = d + R;                        /* fp32 */
    float t = u * s;                        /* fp32 */
    t = t + 0.5f;                           /* fp32 */
    float qf = floorf(t);
    int64_t qi = (int64_t)qf;
    if (qi < 0) qi = 0;
    if (qi > L) qi = L;
    /* eq. 6: deltaQ_i = 2 tau R q_i - R ;  Q_m(theta^k)_i = h_i + deltaQ_i */
    float dq = (float)qi * step;            /* fp32 */
    dq = dq - R;                            /* fp32 */
    float hn = h[i] + dq;                   /* fp32 */
    /* eps_i = grad_i - Q_m(theta^k)_i, taken against the stored value */
    float e = g[i] - hn;                    /* fp32 */
    if (q) q[i] = (uint32_t)qi;
    if (delta) delta[i] = dq;
    if (h_new) h_new[i] = hn;
    int64_t c = 2 * qi - L;
    Sq += c * c;
    float nf = rintf(ldexpf(e, K - x));     /* round-half-even to 2^(x-K) */
    int64_t n = (int64_t)nf;
    N += (uint64_t)(n * n);
  }
  if (Sq_out) *Sq_out = Sq;
  if (E2_out) *E2_out = ldexp((double)N, 2 * (x - K));
  if (lhs_out) {
    /* ||2 tau R q - R 1||^2 = (R/L)^2 sum (2 q_i - L)^2 */
    double r = (double)R / (double)L;
    *lhs_out = (r * r) * (double)Sq;
  }
  return LAQ_ORACLE_OK;
}

void laq_oracle_pack(const uint32_t* q, int64_t p, int32_t b, uint32_t* words,
                     int64_t n_words) {
  memset(words, 0, (size_t)n_words * sizeof(uint32_t));
  for (int64_t i = 0; i < p; ++i) {
    for (int32_t k = 0; k < b; ++k) {
      int64_t bit = i * (int64_t)b + k;
      if ((q[i] >> k) & 1u) words[bit >> 5] |= (uint32_t)1 << (bit & 31);
    }
  }
}

void laq_oracle_unpack(const uint32_t* words, int64_t p, int32_t b, uint32_t* q) {
  for (int64_t i = 0; i < p; ++i) {
    uint32_t v = 0;
    for (int32_t k = 0; k < b; ++k) {
      int64_t bit = i * (int64_t)b + k;
      v |= ((words[bit >> 5] >> (bit & 31)) & 1u) << k;
    }
    q[i] = v;
  }
}

void laq_oracle_dequantize(const uint32_t* q, int64_t p, int32_t b, float R,
                           float* delta) {
  const float Lf = (float)(((int64_t)1 << b) - 1);
  const float two_R = 2.0f * R;
  const float s = Lf / two_R;
  const float step = two_R / Lf;
  if (R == 0.0f || !isfinite(s)) {
    for (int64_t i = 0; i < p; ++i) delta[i] = 0.0f;
    return;
  }
  for (int64_t i = 0; i < p; ++i) {
    float dq = (float)q[i] * step;          /* fp32 */
    delta[i] = dq - R;                      /* fp32 */
  }
}

int laq_oracle_skip(double lhs, double E2, double Ehat2, const double* xi,
                    const double* dtheta2, int32_t D, float alpha, int32_t M,
                    int32_t t_m, int32_t t_bar, double* rhs_out) {
  /* (7a) right-hand side, fp64, left-to-right */
  double Hsum = 0.0;
  for (int32_t d = 0; d < D; ++d) {
    double term = xi[d] * dtheta2[d];
    Hsum = (d == 0) ? term : Hsum + term;
  }
  double a2 = (double)alpha * (double)alpha;
  double m2 = (double)M * (double)M;
  double c = 1.0 / (a2 * m2);
  double err = E2 + Ehat2;
  double rhs = c * Hsum + 3.0 * err;
  if (rhs_out) *rhs_out = rhs;
  /* (7b): an upload is forced once the clock has reached t_bar */
  return (t_m < t_bar) && (lhs <= rhs);
}

double laq_oracle_server(const float* delta, const uint8_t* upload, int32_t M,
                         int64_t p, float alpha, float* nabla, float* theta) {
  double n2 = 0.0;
  for (int64_t i = 0; i < p; ++i) {
    float acc = 0.0f;
    for (int32_t m = 0; m < M; ++m)
      if (upload[m]) acc = acc + delta[(int64_t)m * p + i];   /* fp32 */
    float nb = nabla[i] + acc;                                /* fp32 */
    nabla[i] = nb;
    float st = alpha * nb;                                    /* fp32 */
    theta[i] = theta[i] - st;                                 /* fp32 */
    n2 += (double)nb * (double)nb;
  }
  return ((double)alpha * (double)alpha) * n2;
}

int laq_oracle_iteration(int32_t M, int64_t p, int32_t b, int32_t D,
                         const double* xi, int32_t t_bar, float alpha,
                         const float* G, float* H, float* nabla, float* theta,
                         double* Ehat2, int32_t* t, double* dtheta2,
                         uint64_t* uploads, uint64_t* bits_total, float* R,
                         uint32_t* q, uint8_t* upload, int64_t* Sq, double* E2,
                         double* lhs, double* rhs, int32_t force_upload) {
  if (M < 1 || p < 1 || D < 1) return LAQ_ORACLE_EINVAL;
  float* delta = (float*)malloc((size_t)M * (size_t)p * sizeof(float));
  float* h_new = (float*)malloc((size_t)M * (size_t)p * sizeof(float));
  uint8_t* up = (uint8_t*)malloc((size_t)M);
  double* e2 = (double*)malloc((size_t)M * sizeof(double));
  int* st = (int*)malloc((size_t)M * sizeof(int));
  if (!delta || !h_new || !up || !e2 || !st) {
    free(delta); free(h_new); free(up); free(e2); free(st);
    return LAQ_ORACLE_EINVAL;
  }

  /* Algorithm 2, worker loop: workers are independent of one another */
#pragma omp parallel for schedule(dynamic, 1)
  for (int32_t m = 0; m < M; ++m) {
    const float* g = G + (int64_t)m * p;
    float* h = H + (int64_t)m * p;
    float Rm; int64_t Sqm; double E2m, lhsm, rhsm;
    st[m] = laq_oracle_quantize(g, h, p, b, &Rm, q ? q + (int64_t)m * p : NULL,
                                delta + (int64_t)m * p, h_new + (int64_t)m * p,
                                &Sqm, &E2m, &lhsm);
    if (st[m] != LAQ_ORACLE_OK) { up[m] = 0; e2[m] = 0.0; continue; }
    int skip = laq_oracle_skip(lhsm, E2m, Ehat2[m], xi, dtheta2, D, alpha, M,
                               t[m], t_bar, &rhsm);
    if (force_upload) skip = 0;
    up[m] = (uint8_t)!skip;
    e2[m] = E2m;
    if (R) R[m] = Rm;
    if (Sq) Sq[m] = Sqm;
    if (E2) E2[m] = E2m;
    if (lhs) lhs[m] = lhsm;
    if (rhs) rhs[m] = rhsm;
  }
  int status = LAQ_ORACLE_OK;
  for (int32_t m = 0; m < M; ++m)
    if (st[m] != LAQ_ORACLE_OK) status = st[m];
  if (status == LAQ_ORACLE_OK) {
    const uint64_t msg_bits = (b == LAQ_ORACLE_B_EXACT)
                                  ? (uint64_t)32 * (uint64_t)p
                                  : (uint64_t)32 + (uint64_t)b * (uint64_t)p;
    for (int32_t m = 0; m < M; ++m) {
      if (up[m]) {
        /* upload: theta_hat_m = theta^k, so the stored Q_m becomes h + deltaQ */
        memcpy(H + (int64_t)m * p, h_new + (int64_t)m * p, (size_t)p * sizeof(float));
        Ehat2[m] = e2[m];
        t[m] = 0;
        if (uploads) uploads[m] += 1;
        if (bits_total) *bits_total += msg_bits;
      } else {
        t[m] += 1;
      }
      if (upload) upload[m] = up[m];
    }
    /* server: eq. 4, then push ||theta^{k+1}-theta^k||^2 to the history */
    double d2 = laq_oracle_server(delta, up, M, p, alpha, nabla, theta);
    for (int32_t d = D - 1; d > 0; --d) dtheta2[d] = dtheta2[d - 1];
    dtheta2[0] = d2;
  }
  free(delta); free(h_new); free(up); free(e2); free(st);
  return status;
}
