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

// ------------------------------------------------------------------ multinomial logistic regression on the matrix cores
//
// Both products of the softmax-regression gradient are skinny GEMMs:
//   Z[16 rows][C] = X[16][F] Theta^T        and        Gacc[C][F] += R^T[C][16] X[16][F].
// They map onto v_mfma_f32_16x16x4_f32 with the class dimension padded to 16.
// One block of 16 wavefronts owns a range of rows and walks it in tiles of 16
// rows.  Tiles are copied once from HBM to LDS (coalesced, prefetched into
// registers two tiles ahead, double-buffered in LDS).  For the logits the
// waves split the feature dimension -- wave w always multiplies chunks
// w, w+16, ..., so its fragments of Theta stay in registers for the whole
// kernel -- and their partial products are summed through LDS.  The softmax
// of tile n runs on 4 waves while the other 12 already form the logits of
// tile n+1.  For the rank-16 update the waves split the feature tiles and keep
// their part of Gacc in registers for the whole row range.  LDS allows one
// block per CU, hence the wide block (4 waves per SIMD).
typedef float floatx4 __attribute__((ext_vector_type(4)));
constexpr int kRT = 16;          // rows per tile
constexpr int kSmxWaves = 16;

template <int TMAX>
__global__ __launch_bounds__(64 * kSmxWaves) void softmax_grad_mfma_kernel(
    const float* __restrict__ theta, const float* __restrict__ X, const int32_t* __restrict__ y,
    int64_t N_m, int64_t ldx, int32_t F, int32_t C, int32_t rows_per_block, int32_t ldsF,
    float* __restrict__ part) {
  constexpr int NW = kSmxWaves, NT = 64 * NW;
  extern __shared__ __attribute__((aligned(16))) float smem[];
  float* Xs0 = smem;                         // [16][ldsF]
  float* Xs1 = Xs0 + kRT * ldsF;
  float* Zp0 = Xs1 + kRT * ldsF;             // [NW][16][16] partial logits, two buffers
  float* Zp1 = Zp0 + NW * 256;
  float* Rs = Zp1 + NW * 256;                // [16][16] residuals P - Y
  int* Ys = reinterpret_cast<int*>(Rs + 256);  // [2][16] labels, indexed like the X buffers

  const int m = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, lq = lane >> 4;
  const float* Xm = X + (int64_t)m * N_m * ldx;
  const int32_t* ym = y + (int64_t)m * N_m;
  const int nchunk = (F + 15) / 16, FP = nchunk * 16, nf4 = FP / 4;

  // Theta fragments of this wave's feature chunks (B operand of the logits): lane
  // (class j = l16, quarter lq) holds Theta[j][16 t + 4 lq .. +3], zero past C or F.
  // They go through LDS (staged in the first tile buffer) rather than straight
  // from global memory into registers: the matrix instructions of the main loop
  // then depend on LDS counters only and never wait behind the tile prefetch.
  for (int idx = tid; idx < kRT * FP; idx += NT) {
    const int c = idx / FP, f = idx - c * FP;
    Xs0[c * ldsF + f] = (c < C && f < F) ? theta[(int64_t)c * F + f] : 0.0f;
  }
  __syncthreads();
  float4 thf[TMAX];
#pragma unroll
  for (int n = 0; n < TMAX; ++n) {
    const int t = wave + NW * n;
    thf[n] = t < nchunk ? *reinterpret_cast<const float4*>(&Xs0[l16 * ldsF + 16 * t + 4 * lq])
                        : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  __syncthreads();

  const int64_t r_begin = (int64_t)blockIdx.x * rows_per_block;
  int64_t r_end = r_begin + rows_per_block;
  if (r_end > N_m) r_end = N_m;
  const int64_t last_row = r_end - 1;

  // Tile prefetch: PF unconditional 16-byte loads per lane (row and column
  // clamped into the matrix; rows are padded to ldx, a multiple of 4, so a
  // float4 that starts below F stays inside its row); rows >= r_end and columns
  // >= F are zeroed when the registers are written to LDS.
  constexpr int PF = (kRT * NW * TMAX * 16 / 4 + NT - 1) / NT;
  float4 pre[PF];
  int ypre = 0;
  auto gload = [&](int64_t r0) {
    if (tid < kRT) ypre = ym[(r0 + tid < r_end) ? r0 + tid : last_row];
#pragma unroll
    for (int q = 0; q < PF; ++q) {
      int idx = tid + NT * q;
      idx = idx < kRT * nf4 ? idx : kRT * nf4 - 1;
      const int row = idx / nf4;
      int f = (idx - row * nf4) * 4;
      f = f < F ? f : 0;
      int64_t gr = r0 + row;
      gr = gr < r_end ? gr : last_row;
      pre[q] = *reinterpret_cast<const float4*>(Xm + gr * ldx + f);
    }
  };
  auto lstore = [&](float* buf, int which, int64_t r0) {
    if (tid < kRT) Ys[which * kRT + tid] = ypre;
#pragma unroll
    for (int q = 0; q < PF; ++q) {
      const int idx = tid + NT * q;
      if (idx < kRT * nf4) {
        const int row = idx / nf4, f = (idx - row * nf4) * 4;
        const bool rv = r0 + row < r_end;
        float4 v = pre[q];
        v.x = (rv && f < F) ? v.x : 0.0f;
        v.y = (rv && f + 1 < F) ? v.y : 0.0f;
        v.z = (rv && f + 2 < F) ? v.z : 0.0f;
        v.w = (rv && f + 3 < F) ? v.w : 0.0f;
        *reinterpret_cast<float4*>(&buf[row * ldsF + f]) = v;
      }
    }
  };
  // logits of the tile in Xs: partial products of this wave's chunks -> Zp[wave]
  auto logits = [&](const float* Xs, float* Zp) {
    // two accumulators: a dependent chain of these matrix instructions issues at about half rate
    floatx4 acc1 = floatx4{0.f, 0.f, 0.f, 0.f}, acc1b = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int n = 0; n < TMAX; ++n) {
      const int t = wave + NW * n;
      if (t < nchunk) {
        const float4 a = *reinterpret_cast<const float4*>(&Xs[l16 * ldsF + 16 * t + 4 * lq]);
        acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a.x, thf[n].x, acc1, 0, 0, 0);
        acc1b = __builtin_amdgcn_mfma_f32_16x16x4f32(a.y, thf[n].y, acc1b, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a.z, thf[n].z, acc1, 0, 0, 0);
        acc1b = __builtin_amdgcn_mfma_f32_16x16x4f32(a.w, thf[n].w, acc1b, 0, 0, 0);
      }
    }
    acc1 = acc1 + acc1b;
#pragma unroll
    for (int r = 0; r < 4; ++r) Zp[wave * 256 + (4 * lq + r) * 16 + l16] = acc1[r];
  };

  floatx4 acc2[TMAX];
#pragma unroll
  for (int n = 0; n < TMAX; ++n) acc2[n] = floatx4{0.f, 0.f, 0.f, 0.f};

  // prologue: tile 0 in Xs0 with its logits in Zp0, tile 1 in Xs1
  gload(r_begin);
  lstore(Xs0, 0, r_begin);
  const bool have1 = r_begin + kRT < r_end;
  if (have1) gload(r_begin + kRT);
  __syncthreads();
  logits(Xs0, Zp0);
  if (have1) lstore(Xs1, 1, r_begin + kRT);
  __syncthreads();

  int cur = 0;
  for (int64_t r0 = r_begin; r0 < r_end; r0 += kRT) {
    float* Xc = cur ? Xs1 : Xs0;
    float* Xn = cur ? Xs0 : Xs1;
    float* Zc = cur ? Zp1 : Zp0;
    float* Zn = cur ? Zp0 : Zp1;
    const bool more1 = r0 + kRT < r_end;          // tile n+1 exists (already in Xn)
    const bool more2 = r0 + 2 * kRT < r_end;      // tile n+2 exists
    if (more2) gload(r0 + 2 * kRT);

    // softmax of tile n on waves 0..3 (lane = row i, class j), logits of tile n+1 on all
    if (tid < 256) {
      const int i = tid >> 4, j = tid & 15;
      float z = Zc[tid];
#pragma unroll
      for (int wv = 1; wv < NW; ++wv) z += Zc[wv * 256 + tid];
      const bool valid = j < C;
      float zm = valid ? z : -INFINITY;
#pragma unroll
      for (int off = 8; off > 0; off >>= 1) zm = fmaxf(zm, __shfl_xor(zm, off));
      const float e = valid ? expf(z - zm) : 0.0f;
      float den = e;
#pragma unroll
      for (int off = 8; off > 0; off >>= 1) den += __shfl_xor(den, off);
      float rv = 0.0f;
      if (valid && r0 + i < r_end) rv = e / den - (j == Ys[cur * kRT + i] ? 1.0f : 0.0f);
      Rs[tid] = rv;
    }
    if (more1) logits(Xn, Zn);
    __syncthreads();

    // rank-16 update with tile n: wave w owns feature tiles ft = w, w+NW, ...
    float ar[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) ar[u] = Rs[(4 * u + lq) * 16 + l16];
#pragma unroll
    for (int n = 0; n < TMAX; ++n) {
      const int ft = wave + NW * n;
      if (ft < nchunk) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const float b = Xc[(4 * u + lq) * ldsF + 16 * ft + l16];
          acc2[n] = __builtin_amdgcn_mfma_f32_16x16x4f32(ar[u], b, acc2[n], 0, 0, 0);
        }
      }
    }
    __syncthreads();                               // tile n fully consumed: its buffer is free
    if (more2) lstore(Xc, cur, r0 + 2 * kRT);
    __syncthreads();
    cur ^= 1;
  }

  float* out = part + ((int64_t)m * gridDim.x + blockIdx.x) * ((int64_t)C * F);
#pragma unroll
  for (int n = 0; n < TMAX; ++n) {
    const int f = 16 * (wave + NW * n) + l16;
    if (f < F) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int c = 4 * lq + r;
        if (c < C) out[(int64_t)c * F + f] = acc2[n][r];
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

// G[m][i] = (sum over blocks, ascending) part[m][blk][i] / N + (N_m/N) lambda theta[i].
// Also leaves max_i |G[m][i] - H[m][i]| over this block's coordinates (raw bits)
// in rprod[m][blockIdx.x]: the quantizer's radius without another pass over G.
__global__ __launch_bounds__(kThreads) void finish_grad_kernel(const float* __restrict__ part,
                                                               const float* __restrict__ theta,
                                                               int64_t p, int64_t p_stride, int32_t n_blk,
                                                               float inv_N, float reg,
                                                               float* __restrict__ G,
                                                               const float* __restrict__ H,
                                                               uint32_t* __restrict__ rprod) {
  const int m = blockIdx.y;
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  uint32_t mx = 0;
  if (i < p) {
    const float* pm = part + (int64_t)m * n_blk * p;
    float s = 0.0f;
#pragma unroll 8
    for (int k = 0; k < n_blk; ++k) s += pm[(int64_t)k * p + i];
    const float g = fmaf(s, inv_N, reg * theta[i]);
    G[(int64_t)m * p_stride + i] = g;
    mx = __float_as_uint(g - H[(int64_t)m * p_stride + i]) & 0x7fffffffu;
  }
  __shared__ uint32_t sm[kWaves];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const uint32_t o = (uint32_t)__shfl_xor((int)mx, off);
    mx = mx > o ? mx : o;
  }
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = mx;
  __syncthreads();
  if (threadIdx.x == 0)
    rprod[(int64_t)m * gridDim.x + blockIdx.x] = max(max(sm[0], sm[1]), max(sm[2], sm[3]));
}

// ------------------------------------------------------------------ host side

// LDS layout of the matrix-core softmax kernel: row stride (floats) and bytes; 0 if it does not fit.
static size_t softmax_mfma_lds(const laq_ctx* ctx, int* ldsF_out) {
  if (ctx->kind != LAQ_MODEL_SOFTMAX || ctx->C > 16) return 0;
  const int FP = (ctx->F + 15) / 16 * 16;
  if (FP > 16 * kSmxWaves * 4) return 0;
  const int pad = (20 - FP % 32 + 32) % 32;       // row stride = 20 (mod 32) banks: conflict-free b128 reads
  const int ldsF = FP + pad;
  if (ldsF_out) *ldsF_out = ldsF;
  const size_t bytes = ((size_t)2 * kRT * ldsF + (2 * kSmxWaves + 1) * 256 + 2 * kRT) * sizeof(float);
  return bytes <= 160 * 1024 ? bytes : 0;
}

static int logistic_blocks(const laq_ctx* ctx, int64_t N_m, int* rows_per_block) {
  if (softmax_mfma_lds(ctx, nullptr)) {
    // one block per CU at most (LDS-bound occupancy), whole row tiles per block
    const int RT = kRT;
    int64_t want = ctx->n_cu / ctx->M;
    if (want < 1) want = 1;
    const int64_t tiles = (N_m + RT - 1) / RT;
    if (want > tiles) want = tiles;
    const int64_t tpb = (tiles + want - 1) / want;
    *rows_per_block = (int)(tpb * RT);
    return (int)((tiles + tpb - 1) / tpb);
  }
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
    const size_t part = ((size_t)ctx->M * nb * ctx->p * sizeof(float) + 255) & ~(size_t)255;
    const size_t fblocks = (size_t)((ctx->p + kThreads - 1) / kThreads);
    return part + (size_t)ctx->M * fblocks * sizeof(uint32_t);
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
  int ldsF = 0;
  const size_t mfma_lds = softmax_mfma_lds(ctx, &ldsF);
  if (mfma_lds) {
    const int nchunk = (ctx->F + 15) / 16;
#define LAQ_SMM(T)                                                                                     \
  do {                                                                                                 \
    auto kfn = softmax_grad_mfma_kernel<T>;                                                            \
    LAQ_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),                               \
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)mfma_lds));      \
    hipLaunchKernelGGL(kfn, grid, dim3(64 * kSmxWaves), mfma_lds, ctx->stream, theta, ctx->X, ctx->y,   \
                       ctx->N_m, ctx->ldx, ctx->F, ctx->C, rpb, ldsF, part);                            \
  } while (0)
    if (nchunk <= kSmxWaves) LAQ_SMM(1);
    else if (nchunk <= 2 * kSmxWaves) LAQ_SMM(2);
    else LAQ_SMM(4);
#undef LAQ_SMM
  } else if (ctx->kind == LAQ_MODEL_SOFTMAX) {
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
  const size_t part_bytes = ((size_t)ctx->M * nb * ctx->p * sizeof(float) + 255) & ~(size_t)255;
  ctx->rprod = reinterpret_cast<uint32_t*>(ctx->model_ws + part_bytes);
  ctx->rprod_stride = ctx->rprod_count = (int32_t)fgrid.x;
  hipLaunchKernelGGL(finish_grad_kernel, fgrid, dim3(kThreads), 0, ctx->stream, part, theta, ctx->p,
                     ctx->p_stride, nb, inv_N, reg, G, ctx->H, ctx->rprod);
  LAQ_HIP(ctx, hipGetLastError());
  return LAQ_OK;
}

}  // namespace laq
