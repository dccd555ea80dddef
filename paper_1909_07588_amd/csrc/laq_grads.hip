// Worker gradients g_m = grad f_m(theta^k) (Algorithm 2, worker step) for the
// logistic models of the supplement ("Simulation details"): the global loss is
// the mean over all N samples of cross-entropy + (lambda/2)||theta||^2, hence
//     g_m = (1/N) sum_{n in m} grad CE_n(theta) + (N_m/N) lambda theta.
//
// Wave-per-row streaming design: lane l owns features f = l + 64 k.  It keeps
// theta[:, f] and the running gradient for those features in registers, reads
// each sample row once from HBM with fully coalesced 256-byte requests, forms
// the logits with a cross-lane butterfly, and applies the rank-1 update.  No
// LDS traffic in the main loop; partial sums are combined in a fixed order
// (wave -> block -> worker) so results are reproducible run to run.
#include <math.h>

#include "laq_internal.h"

namespace laq {

constexpr int kWaves = kThreads / 64;

__device__ __forceinline__ float wave_allsum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

// ------------------------------------------------------------------ multinomial logistic regression
//
// theta[C][F], P = softmax(theta x), grad CE = (P - onehot(y)) x^T.
// part[m][block][C*F]: un-normalised block sums.
template <int KF, int CMAX>
__global__ __launch_bounds__(kThreads) void softmax_grad_kernel(
    const float* __restrict__ theta, const float* __restrict__ X, const int32_t* __restrict__ y,
    int64_t N_m, int64_t ldx, int32_t F, int32_t C, int32_t rows_per_block, float* __restrict__ part) {
  const int m = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float* Xm = X + (int64_t)m * N_m * ldx;
  const int32_t* ym = y + (int64_t)m * N_m;

  float th[CMAX][KF], acc[CMAX][KF];
#pragma unroll
  for (int c = 0; c < CMAX; ++c)
#pragma unroll
    for (int k = 0; k < KF; ++k) {
      const int f = lane + 64 * k;
      th[c][k] = (c < C && f < F) ? theta[(int64_t)c * F + f] : 0.0f;
      acc[c][k] = 0.0f;
    }

  const int64_t r_begin = (int64_t)blockIdx.x * rows_per_block;
  int64_t r_end = r_begin + rows_per_block;
  if (r_end > N_m) r_end = N_m;

  float xn[KF];
  int64_t r = r_begin + wave;
  if (r < r_end) {
#pragma unroll
    for (int k = 0; k < KF; ++k) {
      const int f = lane + 64 * k;
      xn[k] = (f < F) ? Xm[r * ldx + f] : 0.0f;
    }
  }
  for (; r < r_end; r += kWaves) {
    float x[KF];
#pragma unroll
    for (int k = 0; k < KF; ++k) x[k] = xn[k];
    const int label = ym[r];
    const int64_t rn = r + kWaves;
    if (rn < r_end) {
#pragma unroll
      for (int k = 0; k < KF; ++k) {
        const int f = lane + 64 * k;
        xn[k] = (f < F) ? Xm[rn * ldx + f] : 0.0f;
      }
    }
    float z[CMAX];
#pragma unroll
    for (int c = 0; c < CMAX; ++c) {
      float s = 0.0f;
#pragma unroll
      for (int k = 0; k < KF; ++k) s = fmaf(x[k], th[c][k], s);
      z[c] = s;
    }
#pragma unroll
    for (int c = 0; c < CMAX; ++c)
      if (c < C) z[c] = wave_allsum(z[c]);
    float zmax = z[0];
#pragma unroll
    for (int c = 1; c < CMAX; ++c)
      if (c < C) zmax = fmaxf(zmax, z[c]);
    float den = 0.0f;
#pragma unroll
    for (int c = 0; c < CMAX; ++c)
      if (c < C) { z[c] = expf(z[c] - zmax); den += z[c]; }
    const float inv = 1.0f / den;
#pragma unroll
    for (int c = 0; c < CMAX; ++c) {
      if (c < C) {
        const float rc = z[c] * inv - (c == label ? 1.0f : 0.0f);
#pragma unroll
        for (int k = 0; k < KF; ++k) acc[c][k] = fmaf(rc, x[k], acc[c][k]);
      }
    }
  }

  // block sum in wave order 0,1,2,3 through LDS, then one coalesced store
  __shared__ float red[kWaves - 1][64];
  float* out = part + ((int64_t)m * gridDim.x + blockIdx.x) * ((int64_t)C * F);
#pragma unroll
  for (int c = 0; c < CMAX; ++c) {
#pragma unroll
    for (int k = 0; k < KF; ++k) {
      if (c < C && 64 * k < F) {          // uniform over the block
        if (wave > 0) red[wave - 1][lane] = acc[c][k];
        __syncthreads();
        if (wave == 0) {
          const int f = lane + 64 * k;
          float s = acc[c][k];
          s += red[0][lane];
          s += red[1][lane];
          s += red[2][lane];
          if (f < F) out[(int64_t)c * F + f] = s;
        }
        __syncthreads();
      }
    }
  }
}

// ------------------------------------------------------------------ binary logistic
//
// l = log(1 + exp(-y x.theta)), y in {-1,+1}; dl/dtheta = -y x / (1 + exp(y x.theta)).
template <int KF>
__global__ __launch_bounds__(kThreads) void binlog_grad_kernel(
    const float* __restrict__ theta, const float* __restrict__ X, const int32_t* __restrict__ y,
    int64_t N_m, int64_t ldx, int32_t F, int32_t rows_per_block, float* __restrict__ part) {
  const int m = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float* Xm = X + (int64_t)m * N_m * ldx;
  const int32_t* ym = y + (int64_t)m * N_m;
  float th[KF], acc[KF];
#pragma unroll
  for (int k = 0; k < KF; ++k) {
    const int f = lane + 64 * k;
    th[k] = (f < F) ? theta[f] : 0.0f;
    acc[k] = 0.0f;
  }
  const int64_t r_begin = (int64_t)blockIdx.x * rows_per_block;
  int64_t r_end = r_begin + rows_per_block;
  if (r_end > N_m) r_end = N_m;
  for (int64_t r = r_begin + wave; r < r_end; r += kWaves) {
    float x[KF];
    float s = 0.0f;
#pragma unroll
    for (int k = 0; k < KF; ++k) {
      const int f = lane + 64 * k;
      x[k] = (f < F) ? Xm[r * ldx + f] : 0.0f;
      s = fmaf(x[k], th[k], s);
    }
    s = wave_allsum(s);
    const float yy = (float)ym[r];
    const float coef = -yy / (1.0f + expf(yy * s));
#pragma unroll
    for (int k = 0; k < KF; ++k) acc[k] = fmaf(coef, x[k], acc[k]);
  }
  __shared__ float red[kWaves - 1][64];
  float* out = part + ((int64_t)m * gridDim.x + blockIdx.x) * (int64_t)F;
#pragma unroll
  for (int k = 0; k < KF; ++k) {
    if (64 * k < F) {                     // uniform over the block
      if (wave > 0) red[wave - 1][lane] = acc[k];
      __syncthreads();
      if (wave == 0) {
        const int f = lane + 64 * k;
        float s = acc[k];
        s += red[0][lane];
        s += red[1][lane];
        s += red[2][lane];
        if (f < F) out[f] = s;
      }
      __syncthreads();
    }
  }
}

// G[m][i] = (sum over blocks, ascending) part[m][blk][i] / N + (N_m/N) lambda theta[i]
__global__ __launch_bounds__(kThreads) void finish_grad_kernel(const float* __restrict__ part,
                                                               const float* __restrict__ theta,
                                                               int64_t p, int64_t p_stride, int32_t n_blk,
                                                               float inv_N, float reg,
                                                               float* __restrict__ G) {
  const int m = blockIdx.y;
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= p) return;
  const float* pm = part + (int64_t)m * n_blk * p;
  float s = 0.0f;
  for (int k = 0; k < n_blk; ++k) s += pm[(int64_t)k * p + i];
  G[(int64_t)m * p_stride + i] = fmaf(s, inv_N, reg * theta[i]);
}

// ------------------------------------------------------------------ host side

static int logistic_blocks(const laq_ctx* ctx, int64_t N_m, int* rows_per_block) {
  // about two blocks per CU over all workers, at least 4 rows per wave
  int64_t want = ((int64_t)ctx->n_cu * 2 + ctx->M - 1) / ctx->M;
  int64_t max_by_rows = (N_m + 15) / 16;
  if (want > max_by_rows) want = max_by_rows;
  if (want < 1) want = 1;
  int64_t rpb = (N_m + want - 1) / want;
  *rows_per_block = (int)rpb;
  return (int)((N_m + rpb - 1) / rpb);
}

static bool logistic_supported(const laq_ctx* ctx) {
  const int kf = (ctx->F + 63) / 64;
  if (ctx->kind == LAQ_MODEL_BINLOG) return kf <= 16;
  return kf <= 16 && ctx->C <= 16;
}

size_t mlp_workspace_bytes(const laq_ctx* ctx, int64_t N_m);
int mlp_worker_grads(laq_ctx* ctx, const float* theta, float* G);

size_t model_workspace_bytes(const laq_ctx* ctx, int64_t N_m) {
  if (ctx->kind == LAQ_MODEL_BINLOG || ctx->kind == LAQ_MODEL_SOFTMAX) {
    int rpb;
    const int nb = logistic_blocks(ctx, N_m, &rpb);
    return (size_t)ctx->M * nb * ctx->p * sizeof(float);
  }
  if (ctx->kind == LAQ_MODEL_MLP) return mlp_workspace_bytes(ctx, N_m);
  return 0;
}

template <int KF>
static void launch_softmax(const laq_ctx* ctx, dim3 grid, const float* theta, int rpb, float* part) {
#define LAQ_SM(CM)                                                                                   \
  hipLaunchKernelGGL((softmax_grad_kernel<KF, CM>), grid, dim3(kThreads), 0, ctx->stream, theta, ctx->X, \
                     ctx->y, ctx->N_m, ctx->ldx, ctx->F, ctx->C, rpb, part)
  if (ctx->C <= 4) LAQ_SM(4);
  else if (ctx->C <= 10) LAQ_SM(10);
  else LAQ_SM(16);
#undef LAQ_SM
}

int worker_grads(laq_ctx* ctx, const float* theta, float* G) {
  if (ctx->kind == LAQ_MODEL_MLP) return mlp_worker_grads(ctx, theta, G);
  if (!logistic_supported(ctx))
    return set_error(ctx, LAQ_EINVAL, "logistic models support F <= 1024 and C <= 16 (F=%d, C=%d)", ctx->F, ctx->C);
  int rpb;
  const int nb = logistic_blocks(ctx, ctx->N_m, &rpb);
  float* part = reinterpret_cast<float*>(ctx->model_ws);
  const dim3 grid((unsigned)nb, (unsigned)ctx->M);
  const int kf = (ctx->F + 63) / 64;
  if (ctx->kind == LAQ_MODEL_SOFTMAX) {
    if (kf <= 1) launch_softmax<1>(ctx, grid, theta, rpb, part);
    else if (kf <= 2) launch_softmax<2>(ctx, grid, theta, rpb, part);
    else if (kf <= 4) launch_softmax<4>(ctx, grid, theta, rpb, part);
    else if (kf <= 8) launch_softmax<8>(ctx, grid, theta, rpb, part);
    else if (kf <= 13) launch_softmax<13>(ctx, grid, theta, rpb, part);
    else launch_softmax<16>(ctx, grid, theta, rpb, part);
  } else {
#define LAQ_BL(K)                                                                                      \
  hipLaunchKernelGGL((binlog_grad_kernel<K>), grid, dim3(kThreads), 0, ctx->stream, theta, ctx->X, ctx->y, \
                     ctx->N_m, ctx->ldx, ctx->F, rpb, part)
    if (kf <= 1) LAQ_BL(1);
    else if (kf <= 2) LAQ_BL(2);
    else if (kf <= 4) LAQ_BL(4);
    else if (kf <= 8) LAQ_BL(8);
    else LAQ_BL(16);
#undef LAQ_BL
  }
  const int64_t N = (int64_t)ctx->M * ctx->N_m;
  const float inv_N = (float)(1.0 / (double)N);
  const float reg = (float)(((double)ctx->N_m / (double)N) * (double)ctx->lambda);
  const dim3 fgrid((unsigned)((ctx->p + kThreads - 1) / kThreads), (unsigned)ctx->M);
  hipLaunchKernelGGL(finish_grad_kernel, fgrid, dim3(kThreads), 0, ctx->stream, part, theta, ctx->p,
                     ctx->p_stride, nb, inv_N, reg, G);
  LAQ_HIP(ctx, hipGetLastError());
  return LAQ_OK;
}

}  // namespace laq
