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
#include "laq_tile_loader.h"

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
// rows.  Wave w owns the feature chunks w, w+16, ... of 16 columns in BOTH
// products, so its slice of every tile is private to it:
//   * it loads the slice straight from HBM in the A-operand layout of the
//     logits (lane = row, 4 consecutive columns), two tiles ahead;
//   * the logits' matrix instructions take these registers directly and leave
//     the wave's partial product in LDS (Zp);
//   * the registers are then parked in the wave's own LDS slice, from which the
//     rank-16 update reads them back in its B-operand layout (lane = column);
//     no other wave touches the slice, so no barrier guards it.
// The block meets twice per tile, before and after the softmax, which four
// waves (one per SIMD, each lane holding one of the 256 entries) compute while
// the others wait: on a SIMD, vector and matrix instructions do not run in the
// same cycles, and with other waves' matrix instructions slipping in between
// its dependent vector instructions the softmax took twice as long.  After the
// second barrier every wave forms the logits of the next tile, refills each
// chunk's registers as soon as the chunk is used (a burst of loads stalls the
// waves in the CU's load queue) and goes straight on to the rank update.
// Theta fragments and the wave's part of Gacc stay in registers for the whole
// kernel.  LDS (two slice buffers, two partial-logit buffers: about 135 KB) and
// registers allow one block per CU.
typedef float floatx4 __attribute__((ext_vector_type(4)));
constexpr int kRT = kSmxRowsPerTile;          // rows per tile
constexpr int kSmxWaves = kSmxWavesPerBlock;

// Block barrier that orders LDS accesses only (the waves of the softmax kernel exchange nothing through
// global memory inside the loop): the general __syncthreads() would also wait for every buffer load in
// flight, i.e. for the tiles requested two steps ahead.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// value held by lane (i + N) mod 16 of the same 16-lane row (data-parallel primitive, no LDS)
template <int N>
__device__ __forceinline__ float row_ror(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x120 + N, 0xf, 0xf, false));
}

// GATHER (stochastic variant): the N_m rows the block range walks are the samples
// idx[m][0..N_m) of the worker's shard of N_src rows; the tile loader takes its row from the index
// list (requested one tile further ahead than the rows themselves), so no copy of the drawn
// rows is made.  An index outside the shard is clamped and sets bit 1 of the status word.
// NFULL = nchunk / 16: the chunks w + 16 n, n < NFULL, exist for every wave w and lie wholly inside
// the F columns, so their code is straight-line (no branch, no column mask, LDS and global
// addresses = one lane base + a constant per n); only the chunks n >= NFULL depend on the wave.
//
// SRC says where the rows come from: kSrcRows = the caller's row-major matrix; kSrcGather = the same
// through the index list; kSrcTiled = the tiled copy that tile_rows_kernel writes (a tile one
// contiguous run of nchunk KB, chunk t its t-th KB with lane l's 16 bytes at byte 16 l, zeros past row
// N_m and column F).  From the tiled copy a wave-wide load is one contiguous KB instead of 16 pieces
// of 64 bytes a row apart, which the memory system serves a little faster (42 instead of 44 us on
// the 785-column workload).
constexpr int kSrcRows = 0, kSrcGather = 1, kSrcTiled = 2;

template <int TMAX, int NFULL, int SRC>
__global__ __launch_bounds__(64 * kSmxWaves) void softmax_grad_mfma_kernel(
    const float* __restrict__ theta, const float* __restrict__ X, const int32_t* __restrict__ y,
    int64_t N_m, int64_t N_src, const int32_t* __restrict__ idx, uint32_t* __restrict__ status,
    int64_t ldx, int32_t F, int32_t C, int32_t rows_per_block, float* __restrict__ part) {
  constexpr int NW = kSmxWaves;
  extern __shared__ __attribute__((aligned(16))) float smem[];
  const int m = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // (uniform: branches on it are scalar)
  const int l16 = lane & 15, lq = lane >> 4;
  constexpr bool GATHER = SRC == kSrcGather, TILED = SRC == kSrcTiled;
  const int nchunk = (F + 15) / 16;
  const float* Xm = TILED ? X + (int64_t)m * ((N_src + kRT - 1) / kRT) * ((int64_t)nchunk * 256)
                          : X + (int64_t)m * N_src * ldx;
  const int32_t* ym = y + (int64_t)m * N_src;
  const int32_t* idxm = GATHER ? idx + (int64_t)m * N_m : nullptr;
  float* Xs = smem;                          // [2][nchunk][256]: chunk t belongs to wave t % 16
  float* Zp = Xs + 2 * nchunk * 256;         // [2][NW][64] float4: partial logits in accumulator layout
  float* Rs = Zp + 2 * NW * 256;             // [2][16][16] residuals P - Y

  // Theta fragments (B operand of the logits): lane (class l16, quarter lq) holds
  // Theta[l16][16 t + 4 lq .. +3] for this wave's chunks, zero past C or F.
  float4 thf[TMAX];
#pragma unroll
  for (int n = 0; n < TMAX; ++n) {
    const int f = 16 * (wave + NW * n) + 4 * lq;
    const bool on = l16 < C;
    const float* tp = theta + (int64_t)(on ? l16 : 0) * F;
    float4 v;
    v.x = (on && f < F) ? tp[f < F ? f : 0] : 0.0f;
    v.y = (on && f + 1 < F) ? tp[f + 1 < F ? f + 1 : 0] : 0.0f;
    v.z = (on && f + 2 < F) ? tp[f + 2 < F ? f + 2 : 0] : 0.0f;
    v.w = (on && f + 3 < F) ? tp[f + 3 < F ? f + 3 : 0] : 0.0f;
    thf[n] = v;
  }

  const int64_t r_begin = (int64_t)blockIdx.x * rows_per_block;
  int64_t r_end = r_begin + rows_per_block;
  if (r_end > N_m) r_end = N_m;

  // LDS word of element (row, col) of a 16 x 16 chunk: 16-byte slot 4 rho(row) + (col/4 ^ sigma(row)),
  // rho(row) = row ^ bit 2 of row, sigma(row) = (row / 2) % 4: 16-byte accesses by (row, quarter)
  // lanes and 4-byte accesses by (column, row group) lanes both spread over the banks.
  const int wr_off = ((4 * (l16 ^ ((l16 >> 2) & 1))) + (lq ^ ((l16 >> 1) & 3))) * 4;
  int rd_off[4];                             // matrix instruction u of the update contracts rows 4 u + lq
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int row = 4 * u + lq;
    rd_off[u] = ((4 * (row ^ ((row >> 2) & 1))) + ((l16 >> 2) ^ ((row >> 1) & 3))) * 4 + (l16 & 3);
  }

  // This wave's slice of a tile, HBM -> registers: lane (row l16, quarter lq) takes 16 bytes per
  // chunk.  Rows past r_end are clamped to the last row (their residuals are zero), columns are
  // clamped into the row (rows are padded to ldx, a multiple of 4) and zeroed when consumed.
  const int nf4r = (F + 3) >> 2;
  float4 pre[TMAX];
  // tiled source: the worker's shard as a buffer resource (its loads return zero outside the shard)
  typedef unsigned int uint4v __attribute__((ext_vector_type(4)));
  const uint32_t lane_bytes = 16u * (uint32_t)lane;
  const __amdgpu_buffer_rsrc_t tiled_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<float*>(Xm), 0, TILED ? (int)(((N_src + kRT - 1) / kRT) * (int64_t)nchunk * 1024) : 0, 0x00020000);
  int ypre = 0;
  // GATHER: source rows (entries of the index list) of this lane's tile row and of its softmax row,
  // for the tile the next gload will take; requested one gload earlier
  int ix_next = 0, iy_next = 0;
  auto iload = [&](int64_t r0) {
    if constexpr (GATHER) {
      const int64_t rb = smx_tile_row(r0, r_end);
      const int rows_valid = smx_rows_valid(rb, r_end);
      ix_next = idxm[rb + smx_data_row(l16, rows_valid)];
      iy_next = idxm[rb + smx_label_row(wave, lq, rows_valid)];
    }
  };
  // Where the tile starting at row r0 lies: a per-lane pointer to the lane's 16 bytes of chunk
  // `wave` (chunk w + 16 n lies 1 KB further per n), the pieces for a chunk that may cross column F,
  // and the row of this lane's label.
  struct TileAddr {
    const float* lanep;
    const float* base;
    uint32_t row_off;
    int64_t ysrc;
  };
  auto gaddr = [&](int64_t r0) {
    // uniform tile base + 32-bit lane offsets (few address registers)
    const int64_t rb = smx_tile_row(r0, r_end);               // first row of the tile, clamped
    const int rows_valid = smx_rows_valid(rb, r_end);
    TileAddr A;
    if constexpr (GATHER) {
      int ix = ix_next, iy = iy_next;
      if (ix < 0 || ix >= N_src || iy < 0 || iy >= N_src) {
        atomicOr(status, 2u);
        ix = ix < 0 ? 0 : (ix >= N_src ? (int)N_src - 1 : ix);
        iy = iy < 0 ? 0 : (iy >= N_src ? (int)N_src - 1 : iy);
      }
      A.base = Xm;
      A.row_off = (uint32_t)ix * (uint32_t)ldx;         // (the host checks that a shard has < 2^32 floats)
      A.ysrc = iy;
    } else if constexpr (TILED) {
      A.base = Xm + (rb / kRT) * ((int64_t)nchunk * 256);           // (blocks start on tile boundaries)
      A.row_off = 0;
      A.ysrc = rb + smx_label_row(wave, lq, rows_valid);
      // Byte offset, within the worker's tiled shard, of chunk `wave` of the tile (of chunk 0 for a wave
      // past the tile's last chunk).  It is the same in all lanes: the loads are buffer loads that take
      // it from a scalar register and add the lane's constant 16 l themselves, so no vector instruction
      // computes an address (each one costs this kernel a matrix-instruction slot).
      A.base = Xm;
      A.lanep = Xm;
      A.row_off = smx_tiled_tile_off(rb, nchunk, wave);
      return A;
    } else {
      A.base = Xm + rb * ldx;
      A.row_off = (uint32_t)smx_data_row(l16, rows_valid) * (uint32_t)ldx;
      A.ysrc = rb + smx_label_row(wave, lq, rows_valid);
    }
    A.lanep = A.base + (A.row_off + smx_lane_col(wave, lq));
    return A;
  };
  auto gchunk = [&](int n, const TileAddr& A) {
    if constexpr (TILED) {
      // chunk wave + 16 n lies 16 KB further per n; one past the tile's last chunk reads the wave's first instead
      const uint32_t off = smx_tiled_chunk_off(A.row_off, n, NFULL, wave, nchunk);
      const uint4v v = __builtin_amdgcn_raw_buffer_load_b128(tiled_rsrc, (int)lane_bytes, (int)off, 0);
      return make_float4(__uint_as_float(v[0]), __uint_as_float(v[1]), __uint_as_float(v[2]), __uint_as_float(v[3]));
    }
    if (n < NFULL) return *reinterpret_cast<const float4*>(A.lanep + smx_chunk_step(n));
    return *reinterpret_cast<const float4*>(A.base + (A.row_off + smx_ragged_col(wave, n, lq, nf4r)));
  };

  floatx4 acc2[TMAX];
#pragma unroll
  for (int n = 0; n < TMAX; ++n) acc2[n] = floatx4{0.f, 0.f, 0.f, 0.f};

  // logits of the tile in pre -> Zp[buf][wave]; the tile -> this wave's LDS slice of buffer buf
  // Each chunk's registers are refilled from the tile at `next` as soon as the chunk is used: the
  // 64 loads a CU issues per tile then reach the address unit spread over the whole step (issued in
  // one burst they held every wave at its last load for up to 1.3 us, right before a barrier).
  auto consume = [&](float4 (&pre)[TMAX], int buf, const TileAddr& next) {
    floatx4 za = floatx4{0.f, 0.f, 0.f, 0.f}, zb = floatx4{0.f, 0.f, 0.f, 0.f};
    float* xw = Xs + (buf * nchunk + wave) * 256 + wr_off;     // this lane's 16 bytes of chunk `wave`
#pragma unroll
    for (int n = 0; n < TMAX; ++n) {
      if (n < NFULL) {
        const float4 a = pre[n];
        za = __builtin_amdgcn_mfma_f32_16x16x4f32(a.x, thf[n].x, za, 0, 0, 0);
        zb = __builtin_amdgcn_mfma_f32_16x16x4f32(a.y, thf[n].y, zb, 0, 0, 0);
        za = __builtin_amdgcn_mfma_f32_16x16x4f32(a.z, thf[n].z, za, 0, 0, 0);
        zb = __builtin_amdgcn_mfma_f32_16x16x4f32(a.w, thf[n].w, zb, 0, 0, 0);
        *reinterpret_cast<float4*>(xw + NW * 256 * n) = a;
        pre[n] = gchunk(n, next);
      } else if (wave + NW * n < nchunk) {                    // uniform over the wave
        float4 a = pre[n];
        const int f = 16 * (wave + NW * n) + 4 * lq;
        a.x = f < F ? a.x : 0.0f;
        a.y = f + 1 < F ? a.y : 0.0f;
        a.z = f + 2 < F ? a.z : 0.0f;
        a.w = f + 3 < F ? a.w : 0.0f;
        za = __builtin_amdgcn_mfma_f32_16x16x4f32(a.x, thf[n].x, za, 0, 0, 0);
        zb = __builtin_amdgcn_mfma_f32_16x16x4f32(a.y, thf[n].y, zb, 0, 0, 0);
        za = __builtin_amdgcn_mfma_f32_16x16x4f32(a.z, thf[n].z, za, 0, 0, 0);
        zb = __builtin_amdgcn_mfma_f32_16x16x4f32(a.w, thf[n].w, zb, 0, 0, 0);
        *reinterpret_cast<float4*>(xw + NW * 256 * n) = a;
        pre[n] = gchunk(n, next);
      }
    }
    za = za + zb;
    *reinterpret_cast<floatx4*>(&Zp[((buf * NW + wave) * 64 + lane) * 4]) = za;   // element r: row 4 lq + r, class l16
  };

  // Residuals of rows 4 wave .. 4 wave + 3 (waves 0..3, one per SIMD: every lane holds one of the
  // 256 entries; the vector ALU and the matrix pipe of a SIMD share one issue port, so the softmax
  // must cost as few wave instructions as possible).  Lane (class l16, lq) handles row 4 wave + lq.
  auto softmax_rows = [&](int buf, int64_t r0, int ylab) {
    const int i = 4 * wave + lq;
    const float* Zb = Zp + buf * NW * 256 + (wave * 16 + l16) * 4 + lq;   // element lq of lane (l16, wave)
    float z = Zb[0];
#pragma unroll
    for (int wv = 1; wv < NW; ++wv) z += Zb[wv * 256];
    const bool valid = l16 < C;
    float zm = valid ? z : -INFINITY;
    zm = fmaxf(zm, row_ror<8>(zm));
    zm = fmaxf(zm, row_ror<4>(zm));
    zm = fmaxf(zm, row_ror<2>(zm));
    zm = fmaxf(zm, row_ror<1>(zm));
    const float e = valid ? expf(z - zm) : 0.0f;
    float den = e;
    den += row_ror<8>(den);
    den += row_ror<4>(den);
    den += row_ror<2>(den);
    den += row_ror<1>(den);
    float rv = 0.0f;
    if (valid && r0 + i < r_end) rv = e / den - (l16 == ylab ? 1.0f : 0.0f);
    Rs[buf * 256 + i * 16 + l16] = rv;
  };
  // rank-16 update with the tile parked in buffer buf
  auto rank_update = [&](int buf) {
    const float* xw = Xs + (buf * nchunk + wave) * 256;
    float ar[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) ar[u] = Rs[buf * 256 + (4 * u + lq) * 16 + l16];
    // whole chunks first: their reads are issued together and the matrix instructions of different
    // chunks (independent accumulators) alternate
    float bf[NFULL > 0 ? NFULL : 1][4];
#pragma unroll
    for (int n = 0; n < NFULL; ++n)
#pragma unroll
      for (int u = 0; u < 4; ++u) bf[n][u] = xw[NW * 256 * n + rd_off[u]];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int n = 0; n < NFULL; ++n)
        acc2[n] = __builtin_amdgcn_mfma_f32_16x16x4f32(ar[u], bf[n][u], acc2[n], 0, 0, 0);
#pragma unroll
    for (int n = NFULL; n < TMAX; ++n) {
      if (wave + NW * n < nchunk) {                           // uniform over the wave
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const float b = xw[NW * 256 * n + rd_off[u]];
          acc2[n] = __builtin_amdgcn_mfma_f32_16x16x4f32(ar[u], b, acc2[n], 0, 0, 0);
        }
      }
    }
  };

  // Pipeline for tile n: [barrier: partial logits of tile n complete] waves 0..3 turn them into
  // residuals while the others wait (their matrix instructions would slip in between the dependent
  // vector instructions of the softmax and stretch it threefold); [barrier: residuals complete]
  // every wave forms the logits of tile n+1 from its registers, refilling them chunk by chunk with
  // tile n+2, and goes straight on to the rank update with tile n, whose slice it parked itself one
  // step earlier.  Everything is unconditional: past the block's range the loads are clamped to its
  // last row and the results are never used (under branches the compiler merges register sets with
  // copies and waits for loads right after issuing them: a memory latency per tile).
  if (r_begin >= r_end) return;                     // (uniform; cannot happen with the host's grid)
  iload(r_begin);
  TileAddr A = gaddr(r_begin);
#pragma unroll
  for (int n = 0; n < TMAX; ++n) pre[n] = gchunk(n, A);
  ypre = ym[A.ysrc];
  iload(r_begin + kRT);
  A = gaddr(r_begin + kRT);
  int ycur = ypre;                                  // labels of this lane's softmax row in the tile of Zp[0]
  {
    const int yload = ym[A.ysrc];
    iload(r_begin + 2 * kRT);
    consume(pre, 0, A);
    asm volatile("v_mov_b32 %0, %1" : "=v"(ypre) : "v"(yload));   // (landed before the loop: see below)
  }
  int buf = 0;
  for (int64_t r0 = r_begin; r0 < r_end; r0 += kRT) {
    lds_barrier();                                  // Zp[buf] complete; Zp[buf ^ 1] and slice buffer buf ^ 1 free
    if (wave < 4) softmax_rows(buf, r0, ycur);      // uniform over the wave
    lds_barrier();                                  // Rs[buf] complete
    A = gaddr(r0 + 2 * kRT);
    // The label and index requests go out BEFORE the tile's: a wave waits for a load by counting how
    // many younger ones may still be in flight, so waiting for the youngest request of a step means
    // waiting for all of them.  And the label is moved to its register at the END of the step it was
    // requested in (a wait for all but the four tile loads behind it): left in flight across the
    // loop's back edge it made the compiler wait for every load at the top of the next step, so that
    // the tile requested two steps ahead had to land within the same step.
    const int yload = ym[A.ysrc];
    iload(r0 + 3 * kRT);
    consume(pre, buf ^ 1, A);
    rank_update(buf);
    ycur = ypre;
    asm volatile("v_mov_b32 %0, %1" : "=v"(ypre) : "v"(yload));
    buf ^= 1;
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
// FLY block partials are in flight at a time (16, or 32 when there are more than 16 of them).
template <int FLY>
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
    // FLY block partials in flight (blocks past the last repeat it, unused), added in ascending
    // order; theta and the stored gradient are requested with the first of them
    const float th = theta[i], hq = H[(int64_t)m * p_stride + i];
    for (int k = 0; k < n_blk; k += FLY) {
      float v[FLY];
#pragma unroll
      for (int u = 0; u < FLY; ++u) v[u] = pm[(int64_t)(k + u < n_blk ? k + u : n_blk - 1) * p + i];
#pragma unroll
      for (int u = 0; u < FLY; ++u)
        if (k + u < n_blk) s += v[u];
    }
    const float g = fmaf(s, inv_N, reg * th);
    G[(int64_t)m * p_stride + i] = g;
    mx = __float_as_uint(g - hq) & 0x7fffffffu;
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

// Tiled copy of the bound rows for softmax_grad_mfma_kernel<.., kSrcTiled>: worker m, tile T (16 rows),
// chunk t (16 columns) -> 256 floats at ((m tiles + T) nchunk + t) 256; float 4 l + j of a chunk is
// X[16 T + l % 16][16 t + 4 (l / 16) + j] (the kernel's lane l holds row l % 16, quarter l / 16 of a
// chunk), zero past row N_m or column F.  One thread per 16 bytes.
__global__ __launch_bounds__(kThreads) void tile_rows_kernel(const float* __restrict__ X, int64_t N_m, int64_t ldx,
                                                            int32_t F, int64_t tiles, float* __restrict__ Xt) {
  const int m = blockIdx.y;
  const int nchunk = (F + 15) / 16;
  const int64_t per_worker = tiles * nchunk * 64;            // 16-byte pieces
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= per_worker) return;
  const int l = (int)(i & 63);
  const int64_t c = i >> 6;
  const int t = (int)(c % nchunk);
  const int64_t row = (c / nchunk) * kRT + (l & 15);
  const int f = 16 * t + 4 * (l >> 4);
  float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
  if (row < N_m) {
    const float* xr = X + ((int64_t)m * N_m + row) * ldx;
    if (f < F) v.x = xr[f];
    if (f + 1 < F) v.y = xr[f + 1];
    if (f + 2 < F) v.z = xr[f + 2];
    if (f + 3 < F) v.w = xr[f + 3];
  }
  reinterpret_cast<float4*>(Xt)[(int64_t)m * per_worker + i] = v;
}

// ------------------------------------------------------------------ host side

// LDS bytes of the matrix-core softmax kernel (tile slices, partial logits, residuals); 0 if the
// model does not fit it.
static size_t softmax_mfma_lds(const laq_ctx* ctx) {
  if (ctx->kind != LAQ_MODEL_SOFTMAX || ctx->C > 16) return 0;
  const int nchunk = (ctx->F + 15) / 16;
  if (nchunk > kSmxWaves * 4) return 0;
  const size_t bytes = ((size_t)2 * nchunk * 256 + (2 * kSmxWaves + 2) * 256) * sizeof(float);
  return bytes <= 160 * 1024 ? bytes : 0;
}

static int logistic_blocks(const laq_ctx* ctx, int64_t N_m, int* rows_per_block) {
  if (softmax_mfma_lds(ctx)) {
    // one block per CU at most (LDS-bound occupancy), whole row tiles per block
    return smx_blocks(ctx->n_cu, ctx->M, N_m, rows_per_block);
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

size_t tiled_data_bytes(const laq_ctx* ctx) {
  if (!ctx->X || softmax_mfma_lds(ctx) == 0) return 0;
  const size_t tiles = (size_t)((ctx->N_m + kRT - 1) / kRT), nchunk = (size_t)((ctx->F + 15) / 16);
  // the kernel addresses a worker's tiled shard through a buffer descriptor and 32-bit byte offsets
  if (tiles * nchunk * 1024 >= ((size_t)1 << 32) - ((size_t)1 << 20)) return 0;
  return (size_t)ctx->M * tiles * nchunk * 256 * sizeof(float);
}

int tile_data(laq_ctx* ctx, float* Xt) {
  const int64_t tiles = (ctx->N_m + kRT - 1) / kRT;
  const int64_t pieces = tiles * ((ctx->F + 15) / 16) * 64;
  if ((pieces + kThreads - 1) / kThreads > 0x7fffffffll)
    return set_error(ctx, LAQ_EINVAL, "laq_tile_data: shard too large");
  hipLaunchKernelGGL(tile_rows_kernel, dim3((unsigned)((pieces + kThreads - 1) / kThreads), (unsigned)ctx->M),
                     dim3(kThreads), 0, ctx->stream, ctx->X, ctx->N_m, ctx->ldx, ctx->F, tiles, Xt);
  LAQ_HIP(ctx, hipGetLastError());
  return LAQ_OK;
}

// The matrix-core softmax kernel can take a minibatch's rows straight from the bound data through
// the index list (32-bit float offsets inside a shard).
bool minibatch_reads_in_place(const laq_ctx* ctx) {
  return ctx->kind == LAQ_MODEL_SOFTMAX && softmax_mfma_lds(ctx) != 0 &&
         (uint64_t)ctx->N_m * (uint64_t)ctx->ldx < (1ull << 32);
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
  const size_t mfma_lds = softmax_mfma_lds(ctx);
  if (mfma_lds) {
#define LAQ_SMM(T, NF)                                                                                 \
  do {                                                                                                 \
    auto kfn = ctx->gather_idx ? softmax_grad_mfma_kernel<T, NF, kSrcGather>                           \
               : tiled         ? softmax_grad_mfma_kernel<T, NF, kSrcTiled>                            \
                               : softmax_grad_mfma_kernel<T, NF, kSrcRows>;                            \
    LAQ_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),                               \
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)mfma_lds));      \
    hipLaunchKernelGGL(kfn, grid, dim3(64 * kSmxWaves), mfma_lds, ctx->stream, theta,                   \
                       tiled ? ctx->Xtiled : ctx->X, ctx->y,                                            \
                       ctx->N_m, ctx->gather_idx ? ctx->gather_rows : ctx->N_m, ctx->gather_idx,        \
                       ctx->sc.status, ctx->ldx, ctx->F, ctx->C, rpb, part);                            \
  } while (0)
    // the tiled copy stands for the rows it was made from (a minibatch call binds other rows)
    const bool tiled = ctx->Xtiled && !ctx->gather_idx && ctx->tiled_for == ctx->X && ctx->tiled_rows == ctx->N_m;
    // chunks n < nfull exist for every wave and hold no column >= F (the tiled copy is zero there)
    int tmax, nfull;
    smx_variant(ctx->F, tiled, tmax, nfull);
    if (tmax == 1) { if (nfull >= 1) LAQ_SMM(1, 1); else LAQ_SMM(1, 0); }
    else if (tmax == 2) { if (nfull >= 2) LAQ_SMM(2, 2); else LAQ_SMM(2, 1); }
    else if (nfull >= 4) LAQ_SMM(4, 4);
    else if (nfull == 3) LAQ_SMM(4, 3);
    else LAQ_SMM(4, 2);
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
  if (nb > 16)
    hipLaunchKernelGGL(finish_grad_kernel<32>, fgrid, dim3(kThreads), 0, ctx->stream, part, theta, ctx->p,
                       ctx->p_stride, nb, inv_N, reg, G, ctx->H, ctx->rprod);
  else
    hipLaunchKernelGGL(finish_grad_kernel<16>, fgrid, dim3(kThreads), 0, ctx->stream, part, theta, ctx->p,
                       ctx->p_stride, nb, inv_N, reg, G, ctx->H, ctx->rprod);
  LAQ_HIP(ctx, hipGetLastError());
  return LAQ_OK;
}

}  // namespace laq
