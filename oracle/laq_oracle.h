/*
 * LAQ oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, single-purpose CPU statement of what one LAQ iteration
 * computes (Sun, Chen, Giannakis, Yang: "Communication-Efficient Distributed
 * Learning via Lazily Aggregated Quantized Gradients", Algorithm 2, eqs. 4-7).
 * It exists so that the HIP library can be compared against it; it shares no
 * code with that library and nothing in the product path may call it.
 *
 * Every function takes plain host pointers. Floating-point steps that decide
 * an integer (codes, the skip predicate) are written as explicit single
 * IEEE-754 operations in the order stated beside them; compile with
 * -ffp-contract=off and without -ffast-math so that order is what runs.
 *
 * Parity pins (tests/test_oracle_*.py): brute-force nearest-grid codes in exact
 * rational arithmetic, the error bound of Sec. 2.1, grid membership of deltaQ,
 * power-of-two scale invariance, GD / LAG / QGD reductions (eq. 8 remark),
 * forced-upload window, the bit counts of Tables 2-3, finite differences for
 * the model gradients.  Unpinned: the upload counts / curves / accuracies of
 * Tables 2-3 themselves (they need MNIST and an initialisation the paper does
 * not state).
 */
#ifndef LAQ_ORACLE_H
#define LAQ_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* b == LAQ_ORACLE_B_EXACT selects the identity quantizer (the "b large
 * enough" limit of the remark after eq. 8): Q_m(theta^k) = grad f_m(theta^k). */
#define LAQ_ORACLE_B_EXACT 32

enum {
  LAQ_ORACLE_OK = 0,
  LAQ_ORACLE_EINVAL = 1,
  LAQ_ORACLE_ENONFINITE = 4
};

/* Fixed-point exponent K of the order-free squared-error sum (see
 * laq_oracle_quantize). */
int32_t laq_oracle_eps_K(int64_t p);

/* Number of 32-bit words holding p b-bit codes as one LSB-first bitstream. */
int64_t laq_oracle_code_words(int64_t p, int32_t b);

/*
 * Innovation quantizer of one worker (Sec. 2.1, eqs. 5-6).
 *   g[p]      fresh local gradient  grad f_m(theta^k)
 *   h[p]      last uploaded quantized gradient Q_m(theta_hat_m^{k-1})
 * outputs
 *   *R        radius ||g - h||_inf
 *   q[p]      integer codes in [0, 2^b-1]              (may be NULL)
 *   delta[p]  deltaQ = 2 tau R q - R 1                 (may be NULL)
 *   h_new[p]  Q_m(theta^k) = h + deltaQ                (may be NULL)
 *   *Sq       sum_i (2 q_i - L)^2,  L = 2^b - 1  (exact integer)
 *   *E2       ||eps||_2^2, eps = g - h_new
 *   *lhs      ||deltaQ||_2^2 = (R/L)^2 Sq
 * returns LAQ_ORACLE_OK, or LAQ_ORACLE_ENONFINITE when R or 2R is not finite.
 */
int laq_oracle_quantize(const float* g, const float* h, int64_t p, int32_t b,
                        float* R, uint32_t* q, float* delta, float* h_new,
                        int64_t* Sq, double* E2, double* lhs);

/* Pack codes into the wire format: code i occupies bits [i*b, (i+1)*b) of a
 * little-endian bitstream over uint32 words; unused tail bits are zero.
 * words must hold n_words >= laq_oracle_code_words(p,b) entries; all n_words
 * are written. */
void laq_oracle_pack(const uint32_t* q, int64_t p, int32_t b, uint32_t* words,
                     int64_t n_words);
void laq_oracle_unpack(const uint32_t* words, int64_t p, int32_t b, uint32_t* q);

/* Dequantise a received message (R, q): delta_i = (float(q_i) * step) - R
 * with step = (2R)/L  (eq. 6). */
void laq_oracle_dequantize(const uint32_t* q, int64_t p, int32_t b, float R,
                           float* delta);

/*
 * Skip rule (eqs. 7a, 7b).  dtheta2[d-1] = ||theta^{k+1-d} - theta^{k-d}||^2
 * for d = 1..D.  Returns 1 when the worker skips, 0 when it uploads; writes
 * the right-hand side of (7a) to *rhs when rhs != NULL.
 */
int laq_oracle_skip(double lhs, double E2, double Ehat2, const double* xi,
                    const double* dtheta2, int32_t D, float alpha, int32_t M,
                    int32_t t_m, int32_t t_bar, double* rhs);

/*
 * Server update (eq. 4): acc_i = sum over uploading workers in ascending m
 * of delta[m][i]; nabla_i += acc_i; theta_i -= alpha * nabla_i.
 * delta is [M][p] (rows of skipping workers are ignored).  Returns
 * alpha^2 * ||nabla||^2 (= ||theta^{k+1} - theta^k||^2 in the reals).
 */
double laq_oracle_server(const float* delta, const uint8_t* upload, int32_t M,
                         int64_t p, float alpha, float* nabla, float* theta);

/*
 * One whole LAQ iteration (Algorithm 2 body) on caller-held state, given the
 * fresh gradients G[M][p].  State (all updated in place):
 *   H[M][p], nabla[p], theta[p], Ehat2[M], t[M], dtheta2[D] (index 0 = d=1),
 *   uploads[M], *bits_total.
 * Per-iteration outputs (any may be NULL):
 *   R[M], q[M][p], upload[M] (1 = upload), Sq[M], E2[M], lhs[M], rhs[M].
 * force_upload != 0 ignores the skip rule (Algorithm 1, QGD).
 */
int laq_oracle_iteration(int32_t M, int64_t p, int32_t b, int32_t D,
                         const double* xi, int32_t t_bar, float alpha,
                         const float* G, float* H, float* nabla, float* theta,
                         double* Ehat2, int32_t* t, double* dtheta2,
                         uint64_t* uploads, uint64_t* bits_total, float* R,
                         uint32_t* q, uint8_t* upload, int64_t* Sq, double* E2,
                         double* lhs, double* rhs, int32_t force_upload);

/* ---- model gradients (supplement, "Simulation details") ----------------- */
/* All accumulate over samples in double and round once to float.           */
/* Each returns worker m's share  g_m = (1/N) sum_n grad CE_n + (N_m/N) lambda theta. */

/* Binary logistic loss log(1+exp(-y x.theta)), y in {-1,+1}; X[N_m][ldx]. */
void laq_oracle_grad_binlog(const float* theta, const float* X,
                            const int32_t* y, int64_t N_m, int64_t F,
                            int64_t ldx, int64_t N_total, float lambda,
                            float* g, double* loss_sum);

/* Multinomial logistic regression, theta[C][F], P = softmax(theta x). */
void laq_oracle_grad_softmax(const float* theta, const float* X,
                             const int32_t* y, int64_t N_m, int64_t F,
                             int64_t ldx, int32_t C, int64_t N_total,
                             float lambda, float* g, double* loss_sum);

/* Fully connected ReLU network, dims[0..n_dims-1] = layer widths
 * (dims[0] inputs, dims[n_dims-1] classes); theta = (W_1[in][out], b_1[out],
 * W_2, b_2, ...) flattened; softmax cross-entropy output. */
void laq_oracle_grad_mlp(const float* theta, const float* X, const int32_t* y,
                         int64_t N_m, int64_t ldx, const int32_t* dims,
                         int32_t n_dims, int64_t N_total, float lambda,
                         float* g, double* loss_sum);

int64_t laq_oracle_mlp_params(const int32_t* dims, int32_t n_dims);

/* All M workers' gradients; X is [M][N_m][ldx], y is [M][N_m], G is [M][p].
 * kind: 1 binary logistic (dims = {F}), 2 multinomial logistic
 * (dims = {F, C}), 3 ReLU network (dims = layer widths).  Returns the global
 * loss (1/N) sum_m f_m(theta), regulariser included. */
double laq_oracle_grads_all(int32_t kind, const float* theta, const float* X,
                            const int32_t* y, int32_t M, int64_t N_m,
                            int64_t ldx, const int32_t* dims, int32_t n_dims,
                            float lambda, float* G);

/* Minibatch gradients (SLAQ, Sec. 4): worker m uses the B samples
 * idx[m][0..B) of its shard; g_m = (1/(M B)) sum_j grad CE_{idx[m][j]} +
 * (1/M) lambda theta.  idx is [M][B], values in [0, N_m). */
void laq_oracle_grads_minibatch(int32_t kind, const float* theta, const float* X,
                                const int32_t* y, int32_t M, int64_t N_m,
                                int64_t ldx, const int32_t* dims, int32_t n_dims,
                                float lambda, const int32_t* idx, int64_t B,
                                float* G);

#ifdef __cplusplus
}
#endif
#endif
