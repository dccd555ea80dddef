/*
 * laq.h -- C ABI of the LAQ hot path for AMD Instinct MI355X (gfx950).
 *
 * LAQ = Lazily Aggregated Quantized gradients (Sun, Chen, Giannakis, Yang,
 * NeurIPS 2019).  All M workers of the paper's worker-server protocol are
 * simulated on one GPU.  One iteration of Algorithm 2 is three calls:
 *
 *     laq_worker_grads   g_m = grad f_m(theta^k)                (Alg. 2, worker step)
 *     laq_quantize_skip  (R_m, q_m), upload mask                 (eqs. 5-7)
 *     laq_server_step    nabla^k, theta^{k+1}, stored Q_m        (eq. 4)
 *
 * Conventions
 *  - Every pointer named *_dev is DEVICE memory, every other pointer is HOST
 *    memory.  The library never allocates or frees device memory: state lives
 *    in a caller-provided workspace that must stay alive until laq_destroy.
 *  - All device pointers must be 16-byte aligned.  Per-worker vectors are
 *    rows of a matrix with row stride laq_p_stride(p) floats (gradients,
 *    stored quantized gradients) or laq_w_stride(p, b) 32-bit words (codes).
 *    Padding elements are never read into a result.
 *  - All work is enqueued on the HIP stream given to laq_create; the three
 *    hot calls never synchronise with the host.
 *  - Every call returns a laq_status.  LAQ_EDEVICE means a HIP call failed;
 *    laq_last_error() describes it.  No exception crosses this boundary.
 *  - A context is not thread-safe; calls on one context that overlap in time
 *    (from different host threads or streams) race on its workspace.
 *
 * Finite precision (the paper states its formulas over the reals): codes,
 * radii and upload decisions are a deterministic function of the gradients
 * and the state.  Elementwise steps are single IEEE binary32 operations in
 * the order documented at laq_quantize_skip; the two squared norms that
 * decide an upload are accumulated as exact integers, so they do not depend
 * on the reduction order.
 */
#ifndef LAQ_H
#define LAQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct laq_ctx laq_ctx;

typedef enum laq_status {
  LAQ_OK = 0,
  LAQ_EINVAL = 1,     /* bad argument (null, range, alignment, size)          */
  LAQ_ESTATE = 2,     /* call order: e.g. worker_grads without model and data */
  LAQ_EDEVICE = 3,    /* a HIP runtime call failed                             */
  LAQ_ENONFINITE = 4  /* a radius R_m was inf/NaN (reported by get_counters)  */
} laq_status;

typedef enum laq_model_kind {
  LAQ_MODEL_NONE = 0,    /* caller supplies the gradients                      */
  LAQ_MODEL_BINLOG = 1,  /* binary logistic loss, dims = {F}                   */
  LAQ_MODEL_SOFTMAX = 2, /* multinomial logistic regression, dims = {F, C}     */
  LAQ_MODEL_MLP = 3      /* fully connected ReLU net, dims = layer widths      */
} laq_model_kind;

/* laq_set_mode flags */
#define LAQ_MODE_FORCE_UPLOAD 1u /* every worker uploads every round: Algorithm 1 (QGD) */

#define LAQ_MAX_BITS 16
/* b = LAQ_B_EXACT selects the identity quantizer Q_m(theta^k) = grad f_m(theta^k): the limit of
 * many bits, in which the skip rule (7a) has eps = 0 and LAQ becomes lazy aggregation of exact
 * gradients (LAG); with LAQ_MODE_FORCE_UPLOAD it is plain gradient descent (eq. 2).  The message
 * is g_m itself: codes_dev rows hold its p binary32 words (row stride laq_w_stride(p, 32)), an
 * upload counts 32 p bits, R_dev still reports max |g - h|, and the left side of (7a) is
 * ||g_m - h_m||^2 accumulated in binary64 in a fixed order (exact squares; unlike the integer
 * sums of the b-bit path its last bits depend on that order). */
#define LAQ_B_EXACT 32
#define LAQ_MAX_LAYERS 8

/* Row stride, in floats, of per-worker gradient matrices (p rounded up to a
 * multiple of 4). */
int64_t laq_p_stride(int64_t p);

/* Row stride, in 32-bit words, of the packed code matrix.  Codes of one
 * worker form one LSB-first bitstream over little-endian words: code i sits at
 * bit offset i*b (the 32 + b*p bit message of Sec. 2.1 is this stream plus
 * R_m).  The stride covers ceil(p/8)*b bytes rounded up to 16 bytes; bits
 * past code p-1 inside the first ceil(p*b/32) words are written as zero. */
int64_t laq_w_stride(int64_t p, int32_t b);

/* Bytes of device workspace laq_create needs for these sizes. */
size_t laq_workspace_bytes(int32_t M, int64_t p, int32_t b, int32_t D);

/*
 * Algorithm 2, lines 1-2.  M workers, p parameters, b bits per coordinate
 * (1..16, or LAQ_B_EXACT), D past parameter differences weighted by xi[0..D-1] (host array,
 * xi[d-1] = xi_d >= 0), clock limit t_bar >= D, step size alpha > 0.
 * workspace_dev: at least laq_workspace_bytes(M,p,b,D) bytes, 256-byte
 * aligned, owned by the caller.  hip_stream: a hipStream_t (NULL = the
 * default stream).  Initial state (the paper leaves it open): stored
 * quantized gradients 0, nabla 0, ||eps_hat||^2 = 0, parameter-difference
 * history 0, clocks t_m = t_bar so the first iteration is a full round.
 * On success *out owns a small host object; free it with laq_destroy.
 */
int laq_create(laq_ctx** out, int32_t M, int64_t p, int32_t b, int32_t D,
               const float* xi, int32_t t_bar, float alpha, void* workspace_dev,
               size_t workspace_bytes, void* hip_stream);

int laq_destroy(laq_ctx* ctx);

/* Back to the initial state of laq_create (enqueued on the stream). */
int laq_reset(laq_ctx* ctx);

int laq_set_mode(laq_ctx* ctx, uint32_t flags);

/*
 * Models of the supplement ("Simulation details").  The global loss is the
 * mean over all N = M*N_m samples of cross-entropy + (lambda/2)||theta||^2, so
 * worker m's gradient is (1/N) sum_n grad CE_n + (N_m/N) lambda theta.
 *   BINLOG : dims = {F};      theta[F];    labels in {-1,+1}
 *   SOFTMAX: dims = {F, C};   theta[C][F]; P = softmax(theta x); labels 0..C-1
 *   MLP    : dims = {d_0..d_L}, 2 <= L+1 <= LAQ_MAX_LAYERS+1; theta is
 *            (W_1[d_0][d_1], b_1[d_1], W_2, b_2, ...) flattened, ReLU between
 *            layers, softmax cross-entropy on the last.
 * The parameter count implied by dims must equal p.
 */
int laq_set_model(laq_ctx* ctx, int32_t kind, const int32_t* dims, int32_t n_dims,
                  float lambda);

/* Bytes of device scratch (activations, partial sums) the model needs for
 * N_m samples per worker; 0 if no model is set. */
size_t laq_model_workspace_bytes(const laq_ctx* ctx, int64_t N_m);

/*
 * Training data, caller-owned, device memory: X_dev[M][N_m][ldx] row-major
 * fp32 with ldx >= dims[0], ldx % 4 == 0 (columns past dims[0] are ignored);
 * y_dev[M][N_m] int32.  model_ws_dev: laq_model_workspace_bytes(ctx, N_m)
 * bytes of scratch, 256-byte aligned, caller-owned, alive while used.
 */
int laq_set_data(laq_ctx* ctx, const float* X_dev, const int32_t* y_dev, int64_t N_m,
                 int64_t ldx, void* model_ws_dev, size_t model_ws_bytes);

/*
 * Optional, for the SOFTMAX model.  Worker m evaluates grad f_m on the same
 * local samples in every iteration (Algorithm 2; f_m of eq. 1 is fixed), so
 * the samples can be laid out once for the kernel that reads them in every
 * iteration: laq_tile_data copies the bound X into tiled_dev (caller-owned
 * device memory, 256-byte aligned, at least laq_tiled_data_bytes(ctx) bytes,
 * alive while the data stay bound) as tiles of 16 rows, each one contiguous
 * run of 16-column chunks padded with zeros.  The copy is enqueued on the
 * stream; from then on laq_worker_grads reads tiled_dev instead of X_dev
 * (same arithmetic, same results), and later changes of X_dev are not seen
 * until laq_tile_data is called again.  laq_worker_grads_minibatch keeps
 * reading X_dev, which must stay alive.  laq_set_model and laq_set_data drop
 * the copy.  laq_tiled_data_bytes returns 0 when the bound model and data
 * have no kernel that reads tiles, or a worker's shard would reach 4 GB
 * (then laq_tile_data returns LAQ_EINVAL and the row-major data keep serving).
 */
size_t laq_tiled_data_bytes(const laq_ctx* ctx);
int laq_tile_data(laq_ctx* ctx, void* tiled_dev, size_t tiled_bytes);

/*
 * Algorithm 2, worker step, first half: G_dev[m][0..p) = grad f_m(theta) for
 * all M workers (fp32 arithmetic; row stride laq_p_stride(p)).
 * theta_dev[p] is read only.  Needs laq_set_model and laq_set_data.
 * The kernels that write G also leave max |g - h| per block, so a following
 * laq_quantize_skip on the same G_dev skips its radius pass (one read of G and
 * of the stored gradients less), provided neither the state nor the contents
 * of G_dev change in between.  A caller that edits G_dev in place (clipping,
 * added noise) must withdraw the hand-over with laq_radius_handover(ctx, NULL,
 * NULL, 0) before it calls laq_quantize_skip; the library cannot see such an
 * edit and would quantize with the radius of the gradients as it wrote them.
 */
int laq_worker_grads(laq_ctx* ctx, const float* theta_dev, float* G_dev);

/*
 * Stochastic variant (Sec. 4, "Stochastic gradient-based tests": SLAQ is LAQ
 * run on minibatch gradients).  idx_dev[M][B] int32 (device): worker m uses
 * the B samples idx[m][0..B) of its own shard, indices in [0, N_m), drawn by
 * the caller.  G_dev[m] = (1/(M B)) sum_j grad CE_{idx[m][j]}(theta)
 * + (1/M) lambda theta: the gradient of the loss the minibatches define, an
 * unbiased estimate of the full-batch g_m.  ws_dev: caller-owned scratch of
 * laq_minibatch_workspace_bytes(ctx, B) bytes, 256-byte aligned (gathered
 * rows and the model's scratch for B samples); the data bound by laq_set_data
 * stays bound.  An index outside the shard is clamped and makes
 * laq_get_counters return LAQ_EINVAL.  The radius hand-over to
 * laq_quantize_skip works as for laq_worker_grads; the block maxima it rests
 * on lie in ws_dev, which must therefore stay alive and untouched until the
 * laq_quantize_skip calls on this G_dev have run (or the hand-over is
 * withdrawn).
 */
size_t laq_minibatch_workspace_bytes(const laq_ctx* ctx, int64_t B);
int laq_worker_grads_minibatch(laq_ctx* ctx, const float* theta_dev, const int32_t* idx_dev,
                               int64_t B, void* ws_dev, size_t ws_bytes, float* G_dev);

/*
 * Innovation quantizer (Sec. 2.1, eqs. 5-6) and skip rule (Sec. 2.2, eqs.
 * 7a-7b) for all workers.  With h_m the stored quantized gradient, L = 2^b-1,
 * and (+),(-),(*),(/) single binary32 operations:
 *     d_i = g_i (-) h_i              R_m = max_i |d_i|
 *     s = L (/) (2 (*) R_m)          step = (2 (*) R_m) (/) L
 *     q_i = clamp(floor(((d_i (+) R_m) (*) s) (+) 0.5), 0, L)
 *     delta_i = (q_i (*) step) (-) R_m     eps_i = g_i (-) (h_i (+) delta_i)
 * R_m == 0 (or s not finite) gives q = 0, delta = 0.  The worker skips iff
 *     (R_m/L)^2 sum_i (2 q_i - L)^2  <=  (1/(alpha^2 M^2)) sum_d xi_d dtheta2[d]
 *                                         + 3 (||eps_m||^2 + ||eps_hat_m||^2)
 * and t_m < t_bar (binary64, fixed order), where ||eps_m||^2 is the exact
 * integer sum of rint(eps_i 2^(K-x))^2 scaled by 2^(2(x-K)), 2^(x-1) <= step <
 * 2^x, K = min(20, floor((63 - ceil(log2 p))/2)).
 * Outputs (the "messages"): codes_dev[M][laq_w_stride], R_dev[M],
 * upload_dev[M] (1 = upload, 0 = skip).  Codes and R are written for every
 * worker.  Internal state is not modified except the per-call stash read by
 * laq_server_step, so the call may be repeated.
 */
int laq_quantize_skip(laq_ctx* ctx, const float* G_dev, uint32_t* codes_dev,
                      float* R_dev, uint8_t* upload_dev);

/*
 * For a caller whose own kernel produces the gradients (Sec. 2.1 defines R_m
 * from g_m and the stored Q_m alone, so whoever writes g_m can take the
 * maximum on the way, as laq_worker_grads does): declares that
 * rmax_dev[m * count + i], i < count, hold the raw bits of max |g_j - h_j| over
 * the i-th part of any partition of worker m's coordinates (h = the stored
 * quantized gradients, laq_state_view.H_dev).  Every laq_quantize_skip on the
 * same G_dev then skips its radius pass until the declaration is withdrawn:
 * by laq_server_step, laq_get_state, laq_reset, laq_set_model,
 * laq_worker_grads (which leaves its own), or by this call with count = 0
 * (G_dev and rmax_dev are then ignored).  A laq_quantize_skip on another G_dev
 * in between runs its own radius pass and leaves the declaration intact.  The
 * caller must withdraw it before it changes the contents of G_dev.
 * rmax_dev (device, caller-owned): with count <= 256 it is read by each such
 * laq_quantize_skip and must stay alive and unchanged until then; with count >
 * 256 it is read by a kernel this call enqueues on the stream (the maxima are
 * combined once into the workspace) and may be reused after that.  The values
 * are trusted: if their maximum is not ||g_m - h_m||_inf the codes are those of
 * eq. 5 for that other radius, clamped to [0, L].  count >= 0.
 */
int laq_radius_handover(laq_ctx* ctx, const float* G_dev, const uint32_t* rmax_dev, int32_t count);

/*
 * Server update (eq. 4) and the bookkeeping of Algorithm 2: for workers with
 * upload_dev[m] = 1, in ascending m: delta from (R_m, q_m), stored
 * Q_m += delta, acc_i += delta_i, ||eps_hat_m||^2 = ||eps_m||^2, t_m = 0,
 * uploads_m += 1, bits += 32 + b p; other workers: t_m += 1.  Then
 * nabla_i += acc_i, theta_i -= alpha * nabla_i, and alpha^2 ||nabla||^2 is
 * pushed into the parameter-difference history.  theta_dev[p] is updated in
 * place.  Reads only rows of uploading workers.
 */
int laq_server_step(laq_ctx* ctx, const uint32_t* codes_dev, const float* R_dev,
                    const uint8_t* upload_dev, float* theta_dev);

/*
 * laq_quantize_skip for callers that can neither allocate device memory nor
 * bring scratch for the passes' partial results: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * arithmetic, outputs and radius hand-over as laq_quantize_skip; the block
 * partials of the radius and code passes (maxima of |g - h|, the two integer
 * sums) live in a static device array of the library, 1.3 MB per GPU, held
 * until the process ends, instead of the workspace.  The call allocates
 * nothing.  Limits: M <= 4096 and ceil(p / 2048) <= 512 * floor(65536 / M)
 * (65536 block partials in all, each covering at most 512 tiles of 2048
 * coordinates); larger sizes return LAQ_EINVAL and enqueue nothing.  All
 * contexts on one GPU share that GPU's array: calls of this function that
 * overlap in time on one GPU (different streams or host threads) race on it,
 * even on different contexts.  Every slot a call reads it has written itself,
 * so nothing needs clearing between calls.
 */
int laq_quantize_skip_noalloc(laq_ctx* ctx, const float* G_dev, uint32_t* codes_dev,
                              float* R_dev, uint8_t* upload_dev);

/* Device pointers into the workspace (valid until laq_destroy).  The caller
 * may read or overwrite them between calls with stream-ordered copies; this
 * is how a checkpoint is saved, restored, or a reference state is imposed.
 * Call laq_get_state again before each round of writes: the call also drops
 * the radius that laq_worker_grads may have handed to laq_quantize_skip (it
 * was computed against the stored gradients as they were). */
typedef struct laq_state_view {
  float* H_dev;            /* [M][p_stride] stored Q_m(theta_hat_m)            */
  float* nabla_dev;        /* [p_stride]                                       */
  double* Ehat2_dev;       /* [M] ||eps_hat_m||^2                              */
  int32_t* t_dev;          /* [M] clocks                                       */
  double* dtheta2_dev;     /* [D] index 0 = most recent ||theta^{k+1}-theta^k||^2 */
  int64_t* Sq_dev;         /* [M] last call's sum (2q-L)^2                     */
  double* E2_dev;          /* [M] last call's ||eps_m||^2                      */
  double* lhs_dev;         /* [M] last call's left side of (7a)                */
  double* rhs_dev;         /* [M] last call's right side of (7a)               */
  uint64_t* uploads_dev;   /* [M] upload counts                                */
  uint64_t* bits_dev;      /* [1] total transmitted bits                       */
  uint32_t* status_dev;    /* [1] bit 0: a radius was not finite; bit 1: bad index */
  int64_t p_stride;
  int64_t w_stride;
} laq_state_view;

int laq_get_state(laq_ctx* ctx, laq_state_view* view);

/* Synchronises the stream and copies the counters to host arrays
 * uploads[M], *bits_total.  Returns LAQ_ENONFINITE if any radius so far was
 * not finite, LAQ_EINVAL if a minibatch index was out of range. */
int laq_get_counters(laq_ctx* ctx, uint64_t* uploads, uint64_t* bits_total);

/* Text of the last error on this context ("" if none); owned by the context. */
const char* laq_last_error(const laq_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* LAQ_H */
