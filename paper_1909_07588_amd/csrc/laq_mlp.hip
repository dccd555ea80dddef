// Worker gradients of the fully connected ReLU network (supplement,
// "Simulation details"): forward, softmax cross-entropy, backward, for all M
// workers at once.  theta = (W_1[d0][d1], b_1[d1], W_2, b_2, ...) is shared, so
// the forward products are single GEMMs over all S = M*N_m samples; the
// activation gradients and the weight gradients are GEMMs batched over the
// workers (the first so that its epilogue can leave per-worker bias sums, the
// second written straight into row m of G with the 1/N scale and the
// regulariser share (N_m/N) lambda theta applied in the epilogue).
//
// Dense products run on the fp32 matrix cores: v_mfma_f32_32x32x2_f32 in
// 128x128 block tiles (4 wavefronts of 64x64 each) or 64x64 ones on small
// grids, v_mfma_f32_16x16x4_f32 in 64 x (160..224) tiles for layers that
// narrow.  16-deep K tiles are staged through two LDS buffers, laid out so
// that every operand fetch is a conflict-free ds_read_b32 at an immediate
// offset; the next tile is prefetched into registers while the current one is
// multiplied.  The class layer (C <= 16 columns) is too narrow for these
// tiles and is bandwidth-bound: its own kernels, one read of the activations
// each.
#include <math.h>

#include <type_traits>

#include "laq_internal.h"
#include "laq_tile_loader.h"

namespace laq {

static_assert(kLoaderThreads == kThreads, "the tile map assumes the matrix kernels' block size");

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// One matrix instruction on an MT x MT output tile: 32 x 32 x 2 (16 accumulator registers per lane; lane
// = (k = lane / 32, row or column = lane % 32)) or 16 x 16 x 4 (4 registers; k = lane / 16).
template <int MT> struct MfmaTile;
template <> struct MfmaTile<32> {
  typedef floatx16 Acc;
  static constexpr int kRegs = 16, kStep = 2;
  static __device__ __forceinline__ Acc mma(float a, float b, Acc c) { return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0); }
  // row inside the tile of accumulator register r of a lane in k group kq = a part that depends on the
  // register only + a part that depends on the lane only
  static __device__ __forceinline__ constexpr int row_reg(int r) { return 8 * (r / 4) + (r % 4); }
  static __device__ __forceinline__ int row_lane(int kq) { return 4 * kq; }
  static __device__ __forceinline__ int row(int r, int kq) { return row_reg(r) + row_lane(kq); }
};
template <> struct MfmaTile<16> {
  typedef floatx4 Acc;
  static constexpr int kRegs = 4, kStep = 4;
  static __device__ __forceinline__ Acc mma(float a, float b, Acc c) { return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0); }
  static __device__ __forceinline__ constexpr int row_reg(int r) { return r; }
  static __device__ __forceinline__ int row_lane(int kq) { return 4 * kq; }
  static __device__ __forceinline__ int row(int r, int kq) { return row_reg(r) + row_lane(kq); }
};
// LDS row stride of a K-major tile BX wide: the lanes of one operand read (64 / MT k groups of MT
// consecutive floats, one tile row apart) must spread over the 32 banks two by two
template <int MT> __host__ __device__ constexpr int lds_stride(int BX) {
  return MT == 32 ? BX + 4 : BX + ((16 - BX % 32) + 32) % 32;
}


enum { EPI_BIAS_RELU = 0, EPI_MASK = 1, EPI_GRAD = 2, EPI_PARTIAL = 3 };

struct GemmArgs {
  const float* A;      // TA ? [K][M] : [M][K]
  const float* B;      // [K][N]
  float* C;            // [M][N]
  int32_t M, N, K;
  int64_t lda, ldb, ldc;
  int64_t sA, sB, sC;  // batch strides (elements) for blockIdx.z
  int32_t vecA, vecB;  // operand rows are 16-byte aligned
  const float* aux;    // bias[N] | mask[M][ldaux] (+ blockIdx.z saux) | W[M][ldaux]
  int64_t ldaux, saux;
  // EPI_MASK only: column sums of this block's rows of C (the bias gradient's partial sums), at
  // colpart[(blockIdx.z * gridDim.y + blockIdx.y) * N + column]
  float* colpart;
  float scale, reg;
  // EPI_GRAD only: stored quantized gradients laid out like C, and where to
  // leave this block's max |C - H| (raw bits): rprod[z * rstride + rbase + block]
  const float* Hq;
  uint32_t* rprod;
  int32_t rstride, rbase;
  // split K (EPI_PARTIAL): blockIdx.z = batch * nsplit + split; split s multiplies rows
  // [s ksplit, min(K, (s+1) ksplit)) of the contraction and stores its product at C + z sC
  int32_t nsplit, ksplit;
  // first row of block tiles this launch covers (blockIdx.y counts from it) and the radius slot of its
  // first block: the ragged last rows of the output can be launched on their own, with another tile size
  int32_t y0, slot0;
};

// Tile loaders (tile numbering and the aligned loader's addressing: laq_tile_loader.h).

// K-major source S[k][x]
template <int BX, int BK>
__device__ __forceinline__ void load_direct(const float* S, int64_t ld, int K, int X, int k0, int x0,
                                            int vec, float4 (&r)[TileMap<BX, BK>::NV]) {
  using TM = TileMap<BX, BK>;
#pragma unroll
  for (int i = 0; i < TM::NV; ++i) {
    int kk, xx;
    TM::kmajor((int)threadIdx.x, i, kk, xx);
    const int k = k0 + kk, x = x0 + xx;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (TM::exists((int)threadIdx.x, i) && k < K) {
      const float* src = S + (int64_t)k * ld + x;
      if (vec && x + 3 < X) {
        v = *reinterpret_cast<const float4*>(src);
      } else {
        if (x < X) v.x = src[0];
        if (x + 1 < X) v.y = src[1];
        if (x + 2 < X) v.z = src[2];
        if (x + 3 < X) v.w = src[3];
      }
    }
    r[i] = v;
  }
}
// (PRED: only the float4 whose `on` is set are stored)
template <int BX, int BK, int LD, bool PRED = false>
__device__ __forceinline__ void store_direct(float (*tile)[LD], const float4 (&r)[TileMap<BX, BK>::NV],
                                             const bool* on = nullptr) {
  using TM = TileMap<BX, BK>;
#pragma unroll
  for (int i = 0; i < TM::NV; ++i) {
    int kk, xx;
    TM::kmajor((int)threadIdx.x, i, kk, xx);
    if (TM::exists((int)threadIdx.x, i) && (!PRED || on[i])) *reinterpret_cast<float4*>(&tile[kk][xx]) = r[i];
  }
}

// X-major source S[x][k] (transposed on the way into LDS)
template <int BX, int BK>
__device__ __forceinline__ void load_transposed(const float* S, int64_t ld, int K, int X, int k0, int x0,
                                                int vec, float4 (&r)[TileMap<BX, BK>::NV]) {
  using TM = TileMap<BX, BK>;
#pragma unroll
  for (int i = 0; i < TM::NV; ++i) {
    int kk, xx;
    TM::xmajor((int)threadIdx.x, i, kk, xx);
    const int k = k0 + kk, x = x0 + xx;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (TM::exists((int)threadIdx.x, i) && x < X) {
      const float* src = S + (int64_t)x * ld + k;
      if (vec && k + 3 < K) {
        v = *reinterpret_cast<const float4*>(src);
      } else {
        if (k < K) v.x = src[0];
        if (k + 1 < K) v.y = src[1];
        if (k + 2 < K) v.z = src[2];
        if (k + 3 < K) v.w = src[3];
      }
    }
    r[i] = v;
  }
}
// The LDS image of an operand that arrives X-major keeps the k of a pair (2j, 2j+1) side by side:
// element (k, x) at ((k / 2) BX + x) 2 + k % 2.  A lane's float4 (four k of one x) goes in as two 8-byte
// stores instead of four 4-byte ones, the 64 lanes of a matrix-instruction operand read (k and k + 1, or
// the k groups of a 16 x 16 x 4 instruction, of MT consecutive x) touch consecutive words, and no
// padding is needed for either.
template <int BX, int BK, bool PRED = false>
__device__ __forceinline__ void store_transposed(float* tile, const float4 (&r)[TileMap<BX, BK>::NV],
                                                 const bool* on = nullptr) {
  using TM = TileMap<BX, BK>;
#pragma unroll
  for (int i = 0; i < TM::NV; ++i) {
    int kk, xx;
    TM::xmajor((int)threadIdx.x, i, kk, xx);
    if (TM::exists((int)threadIdx.x, i) && (!PRED || on[i])) {
      *reinterpret_cast<float2*>(&tile[((kk / 2) * BX + xx) * 2]) = make_float2(r[i].x, r[i].y);
      *reinterpret_cast<float2*>(&tile[((kk / 2 + 1) * BX + xx) * 2]) = make_float2(r[i].z, r[i].w);
    }
  }
}

// Aligned operands: unconditional clamped loads (addresses: FastLoaderAddr in laq_tile_loader.h) through
// buffer loads whose base is uniform: the K loop advances it with scalar instructions, the lane offsets
// never change, so no vector instruction is spent on addresses (on a SIMD they take the issue slots the
// matrix instructions need).  The descriptor's size field is left at its maximum: every address is
// clamped into the operand by construction (walked on the host), the hardware check is not relied on.
typedef unsigned int uint4v __attribute__((ext_vector_type(4)));
template <int BX, int BK, bool XMAJOR>
struct FastLoader {
  FastLoaderAddr<BX, BK, XMAJOR> at;
  const float* S;
  static constexpr int NV = FastLoaderAddr<BX, BK, XMAJOR>::NV;
  __device__ __forceinline__ void init(const float* S_, int64_t ld, int K, int X, int x0) {
    S = S_;
    at.init((int)threadIdx.x, ld, K, X, x0);
  }
  static __device__ __forceinline__ float4 load16(const float* base, uint32_t voff) {
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(base), 0, 0xffffffff, 0x00020000);
    const uint4v v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)voff, 0, 0);
    return make_float4(__uint_as_float(v[0]), __uint_as_float(v[1]), __uint_as_float(v[2]), __uint_as_float(v[3]));
  }
  // Loads K tile number `tile`.  Nothing here touches the loaded values, so the wave does not wait
  // for them before it multiplies.
  __device__ __forceinline__ void load(int tile, float4 (&r)[NV]) {
    if (at.is_whole(tile)) {                              // uniform
      const float* base = S + at.base(tile);
#pragma unroll
      for (int i = 0; i < NV; ++i) r[i] = load16(base, at.voff[i]);
    } else {
      const float* base = S + at.partial_base(tile);
#pragma unroll
      for (int i = 0; i < NV; ++i) r[i] = load16(base, at.partial_voff(tile, i));
    }
  }
  // Zeroes what lies outside the operand; called when the registers move to LDS.  KONLY: only the float4
  // past the contraction's end in the last, partial K tile (for a kernel that never stores a float4
  // outside the operand's width and zeroes its LDS cells once, before the K loop).
  template <bool KONLY = false>
  __device__ __forceinline__ void mask(int tile, float4 (&r)[NV]) const {
    if ((KONLY || at.all_in) && at.is_whole(tile)) return;           // uniform: nothing to zero
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const bool ok = at.keep(tile, i);
      float4 v = r[i];
      v.x = ok ? v.x : 0.0f; v.y = ok ? v.y : 0.0f; v.z = ok ? v.z : 0.0f; v.w = ok ? v.w : 0.0f;
      r[i] = v;
    }
  }
};

#ifndef LAQ_GEMM_BK
#define LAQ_GEMM_BK 16
#endif
#ifndef LAQ_GEMM_NBUF
#define LAQ_GEMM_NBUF 2
#endif

// C = op(A) B with a fused epilogue (A: [M][K] or, TA, [K][M]; B: [K][N]).  Four wavefronts in WM rows
// and 4 / WM columns, each with NLM x NLN matrix-instruction tiles of MT x MT: block tile
// MT WM NLM x MT WN NLN.  NBUF = 2: the next K tile is written to the other LDS buffer while the current
// one is multiplied (one barrier per tile).
// RAGGED: an instantiation for blocks on the output's ragged edge: MT x MT sub-tiles that lie wholly
// outside the output take no matrix instructions (their wavefronts still load and stage operands).
template <bool TA, int EPI, int WM, int NLM, int NLN, bool FAST, bool RAGGED = false, int MT = 32>
__device__ __forceinline__ void gemm_body(GemmArgs g) {
  constexpr int BK = LAQ_GEMM_BK, NBUF = LAQ_GEMM_NBUF;
  constexpr int WN = 4 / WM;
  typedef MfmaTile<MT> MM;
  constexpr int KS = MM::kStep;                               // k per matrix instruction
  constexpr int kBM = MT * WM * NLM, kBN = MT * WN * NLN;
  // LDS floats per k of a tile: a padded row for an operand that arrives K-major, BX for one that arrives
  // X-major (pair layout, see store_transposed)
  constexpr int kLdA = TA ? lds_stride<MT>(kBM) : kBM, kLdB = lds_stride<MT>(kBN);
  constexpr int NVA = TileMap<kBM, BK>::NV, NVB = TileMap<kBN, BK>::NV;
  extern __shared__ __attribute__((aligned(16))) float gemm_smem[];
  float (*As)[BK][kLdA] = reinterpret_cast<float (*)[BK][kLdA]>(gemm_smem);
  float (*Bs)[BK][kLdB] = reinterpret_cast<float (*)[BK][kLdB]>(gemm_smem + NBUF * BK * kLdA);
  const float* A = g.A;
  const float* B = g.B;
  if (EPI == EPI_PARTIAL) {
    const int zb = blockIdx.z / g.nsplit, zs = blockIdx.z - zb * g.nsplit;
    const int64_t ks = (int64_t)zs * g.ksplit;
    A += (int64_t)zb * g.sA + (TA ? ks * g.lda : ks);
    B += (int64_t)zb * g.sB + ks * g.ldb;
    g.K = (int32_t)((int64_t)g.K - ks < g.ksplit ? (int64_t)g.K - ks : g.ksplit);
  } else {
    A += (int64_t)blockIdx.z * g.sA;
    B += (int64_t)blockIdx.z * g.sB;
  }
  float* C = g.C + (int64_t)blockIdx.z * g.sC;
  const int ty = (int)blockIdx.y + g.y0;
  const int m0 = ty * kBM, n0 = blockIdx.x * kBN;
  const int lane = threadIdx.x & 63;
  const int wave = RAGGED ? __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)) : (int)(threadIdx.x >> 6);
  const int wy = wave / WN, wx = wave % WN;
  // sub-tiles of this wavefront that hold any output: the first live_m rows of them by the first live_n columns
  int live_m = NLM, live_n = NLN;
  if (RAGGED) {
    live_m = (g.M - m0 - wy * NLM * MT + MT - 1) / MT;
    live_n = (g.N - n0 - wx * NLN * MT + MT - 1) / MT;
    live_m = live_m < 0 ? 0 : (live_m > NLM ? NLM : live_m);
    live_n = live_n < 0 ? 0 : (live_n > NLN ? NLN : live_n);
  }

  typename MM::Acc acc[NLM][NLN];
#pragma unroll
  for (int i = 0; i < NLM; ++i)
#pragma unroll
    for (int j = 0; j < NLN; ++j)
#pragma unroll
      for (int r = 0; r < MM::kRegs; ++r) acc[i][j][r] = 0.0f;

  float4 ra[NVA], rb[NVB];
  FastLoader<kBM, BK, !TA> fa;   // A is [M][K] (row-major in M) unless TA
  FastLoader<kBN, BK, false> fb;
  if (FAST) {
    fa.init(A, g.lda, g.K, g.M, m0);
    fb.init(B, g.ldb, g.K, g.N, n0);
  }
  auto fetch = [&](int k0) {
    if (FAST) {
      fa.load(k0 / BK, ra);
      fb.load(k0 / BK, rb);
      return;
    }
    if (TA) load_direct<kBM, BK>(A, g.lda, g.K, g.M, k0, m0, g.vecA, ra);
    else load_transposed<kBM, BK>(A, g.lda, g.K, g.M, k0, m0, g.vecA, ra);
    load_direct<kBN, BK>(B, g.ldb, g.K, g.N, k0, n0, g.vecB, rb);
  };
  // 16 x 16 tiles (layers 129 to 224 wide: every block tile crosses the operand's edge, and with fewer
  // matrix-instruction cycles per K tile the vector instructions that zero the outside cost 8 % of the
  // issue slots): a float4 outside the operand's width is never stored, its LDS cells are zeroed once.
  constexpr bool EDGE_ONCE = FAST && MT == 16;
  auto stage = [&](int buf, int k0) {
    if (EDGE_ONCE) {
      fa.template mask<true>(k0 / BK, ra);
      fb.template mask<true>(k0 / BK, rb);
      if (TA) store_direct<kBM, BK, kLdA, true>(As[buf], ra, fa.at.xin); else store_transposed<kBM, BK, true>(&As[buf][0][0], ra, fa.at.xin);
      store_direct<kBN, BK, kLdB, true>(Bs[buf], rb, fb.at.xin);
      return;
    }
    if (FAST) {
      fa.mask(k0 / BK, ra);
      fb.mask(k0 / BK, rb);
    }
    if (TA) store_direct<kBM, BK, kLdA>(As[buf], ra); else store_transposed<kBM, BK>(&As[buf][0][0], ra);
    store_direct<kBN, BK, kLdB>(Bs[buf], rb);
  };
  if (EDGE_ONCE) {
    bool offa[NVA], offb[NVB];
    float4 za[NVA], zb[NVB];
#pragma unroll
    for (int i = 0; i < NVA; ++i) { offa[i] = !fa.at.xin[i]; za[i] = make_float4(0.f, 0.f, 0.f, 0.f); }
#pragma unroll
    for (int i = 0; i < NVB; ++i) { offb[i] = !fb.at.xin[i]; zb[i] = make_float4(0.f, 0.f, 0.f, 0.f); }
    for (int buf = 0; buf < NBUF; ++buf) {
      if (TA) store_direct<kBM, BK, kLdA, true>(As[buf], za, offa); else store_transposed<kBM, BK, true>(&As[buf][0][0], za, offa);
      store_direct<kBN, BK, kLdB, true>(Bs[buf], zb, offb);
    }
  }

  fetch(0);
  stage(0, 0);
  __syncthreads();
  const int kh = lane / MT, li = lane % MT;
  // This lane's operand elements of k step 0 in buffer 0, one LDS address per MT x MT tile.  The
  // addresses are made opaque to the compiler: from a common base it pairs two reads into one
  // instruction whose short offsets then need a new base (a vector add) for every k step; from
  // unrelated bases every read is a single instruction with an immediate offset, and the K loop
  // holds no vector instruction for LDS addresses (they cost matrix-instruction issue slots).
  typedef __attribute__((address_space(3))) const float lds_cfloat;
  lds_cfloat* ap[NLM];
  lds_cfloat* bp[NLN];
#pragma unroll
  for (int i = 0; i < NLM; ++i) {
    const int ax = (wy * NLM + i) * MT + li;
    ap[i] = TA ? (lds_cfloat*)&As[0][kh][ax] : (lds_cfloat*)(&As[0][0][0] + ((kh / 2) * kBM + ax) * 2 + kh % 2);
    asm volatile("" : "+v"(ap[i]));
  }
#pragma unroll
  for (int j = 0; j < NLN; ++j) {
    if (MT == 16 && j > 0) {
      bp[j] = bp[0] + j * MT;      // 16 x 16 tiles: one base, immediate offsets (registers are short there)
    } else {
      bp[j] = (lds_cfloat*)&Bs[0][kh][(wx * NLN + j) * MT + li];
      asm volatile("" : "+v"(bp[j]));
    }
  }
  // One K tile: request the next tile, multiply the current one out of LDS buffer CUR, park the next one
  // in the other buffer.  CUR is a compile-time constant (the K loop is unrolled by two), so that the
  // buffers' LDS addresses are immediates.
  auto tile_step = [&](auto cur_c, int k0) {
    constexpr int cur = NBUF == 2 ? decltype(cur_c)::value : 0;
    const bool more = k0 + BK < g.K;
    if (more) fetch(k0 + BK);
    if constexpr (RAGGED) {
      // all operand reads of the K tile first (those of an empty sub-tile stay inside the LDS tile and are
      // not used), then the matrix instructions of the live sub-tiles only (uniform conditions)
      float a1[BK / KS][NLM], b1[BK / KS][NLN];
#pragma unroll
      for (int kk = 0; kk < BK; kk += KS) {
#pragma unroll
        for (int i = 0; i < NLM; ++i) a1[kk / KS][i] = ap[i][(cur * BK + kk) * kLdA];
#pragma unroll
        for (int j = 0; j < NLN; ++j) b1[kk / KS][j] = bp[j][(cur * BK + kk) * kLdB];
      }
#pragma unroll
      for (int i = 0; i < NLM; ++i)
#pragma unroll
        for (int j = 0; j < NLN; ++j)
          if (i < live_m && j < live_n) {
#pragma unroll
            for (int kk = 0; kk < BK; kk += KS)
              acc[i][j] = MM::mma(a1[kk / KS][i], b1[kk / KS][j], acc[i][j]);
          }
    } else if constexpr (MT == 16) {
      // One wavefront row of many small tiles (NLM = 1): registers do not allow a second set of operands,
      // so the column tiles go in two halves and the reads of one half are in flight while the matrix
      // instructions of the other are issued: [reads: half 2 of step s][multiply half 1][reads: half 1 of
      // step s + 1][multiply half 2].
      static_assert(NLM == 1, "16 x 16 tiles: one tile row per wavefront");
      constexpr int H = (NLN + 1) / 2;
      float a1[2], b1[NLN];
      a1[0] = ap[0][(cur * BK) * kLdA];
#pragma unroll
      for (int j = 0; j < H; ++j) b1[j] = bp[j][(cur * BK) * kLdB];
#pragma unroll
      for (int kk = 0; kk < BK; kk += KS) {
        const int s = (kk / KS) & 1;
#pragma unroll
        for (int j = H; j < NLN; ++j) b1[j] = bp[j][(cur * BK + kk) * kLdB];
#pragma unroll
        for (int j = 0; j < H; ++j) acc[0][j] = MM::mma(a1[s], b1[j], acc[0][j]);
        if (kk + KS < BK) {
          a1[s ^ 1] = ap[0][(cur * BK + kk + KS) * kLdA];
#pragma unroll
          for (int j = 0; j < H; ++j) b1[j] = bp[j][(cur * BK + kk + KS) * kLdB];
        }
#pragma unroll
        for (int j = H; j < NLN; ++j) acc[0][j] = MM::mma(a1[s], b1[j], acc[0][j]);
      }
      __builtin_amdgcn_sched_group_barrier(0x100, 1 + H, 0);
#pragma unroll
      for (int kk = 0; kk < BK; kk += KS) {
        __builtin_amdgcn_sched_group_barrier(0x100, NLN - H, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, H, 0);
        if (kk + KS < BK) __builtin_amdgcn_sched_group_barrier(0x100, 1 + H, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, NLN - H, 0);
      }
    } else {
      // the operands of k step s + 1 are requested before the matrix instructions of step s are issued
      float av[2][NLM], bv[2][NLN];
#pragma unroll
      for (int i = 0; i < NLM; ++i) av[0][i] = ap[i][(cur * BK) * kLdA];
#pragma unroll
      for (int j = 0; j < NLN; ++j) bv[0][j] = bp[j][(cur * BK) * kLdB];
#pragma unroll
      for (int kk = 0; kk < BK; kk += KS) {
        const int s = (kk / KS) & 1;
        if (kk + KS < BK) {
#pragma unroll
          for (int i = 0; i < NLM; ++i) av[s ^ 1][i] = ap[i][(cur * BK + kk + KS) * kLdA];
#pragma unroll
          for (int j = 0; j < NLN; ++j) bv[s ^ 1][j] = bp[j][(cur * BK + kk + KS) * kLdB];
        }
#pragma unroll
        for (int i = 0; i < NLM; ++i)
#pragma unroll
          for (int j = 0; j < NLN; ++j)
            acc[i][j] = MM::mma(av[s][i], bv[s][j], acc[i][j]);
      }
      // Instruction order for the scheduler (it would otherwise move every read next to its use to save
      // registers, and the wave would wait out an LDS latency before each group of matrix instructions):
      // reads of step 0; then, per step, the reads of the next step followed by this step's matrix instructions.
      __builtin_amdgcn_sched_group_barrier(0x100, NLM + NLN, 0);
#pragma unroll
      for (int kk = 0; kk < BK; kk += KS) {
        if (kk + KS < BK) __builtin_amdgcn_sched_group_barrier(0x100, NLM + NLN, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, NLM * NLN, 0);
      }
    }
    if (NBUF == 2) {
      // the other buffer was last read before the previous barrier: free to overwrite
      if (more) stage(cur ^ 1, k0 + BK);
      __syncthreads();
    } else {
      __syncthreads();
      if (more) {
        stage(0, k0 + BK);
        __syncthreads();
      }
    }
  };
  for (int k0 = 0; k0 < g.K; k0 += 2 * BK) {
    tile_step(std::integral_constant<int, 0>{}, k0);
    if (k0 + BK < g.K) tile_step(std::integral_constant<int, 1>{}, k0 + BK);
  }

  // epilogue: lane holds C[i][j], j = lane % MT, i = MM::row(r, lane / MT)
  uint32_t dmax = 0;
  const float* Hq = (EPI == EPI_GRAD) ? g.Hq + (int64_t)blockIdx.z * g.sC : nullptr;
  const float* mask = (EPI == EPI_MASK) ? g.aux + (int64_t)blockIdx.z * g.saux : nullptr;
  float csum[NLN];
#pragma unroll
  for (int tj = 0; tj < NLN; ++tj) csum[tj] = 0.0f;
  // Block tiles whose rows all lie inside the output (all but the last row of tiles): every address is block origin (uniform) + lane offset
  // (constant) + an offset that depends on the register only (uniform), which is what a buffer
  // instruction takes as descriptor, vector offset and scalar offset.  Per element that leaves the
  // arithmetic of the epilogue itself; 64-bit row * stride + column per element (quarter-rate multiplies)
  // cost the matrix pipe 2 % of a 2048-deep product and 5 % of a 784-deep one.
  // (columns past the output's width are a per-lane condition that does not change with the register)
  const bool inside = m0 + kBM <= g.M && (int64_t)kBM * g.ldc < (1 << 28) &&
                      (EPI == EPI_BIAS_RELU || EPI == EPI_PARTIAL || (int64_t)kBM * g.ldaux < (1 << 28));
  if (inside) {
    const __amdgpu_buffer_rsrc_t rc =
        __builtin_amdgcn_make_buffer_rsrc(C + (int64_t)m0 * g.ldc + n0, 0, 0xffffffff, 0x00020000);
    const int lrow = wy * NLM * MT + MM::row_lane(kh), lcol = wx * NLN * MT + li;
    const int voc = (lrow * (int)g.ldc + lcol) * 4;
    const int ldc4 = (int)g.ldc * 4;
    if (EPI == EPI_BIAS_RELU) {
#pragma unroll
      for (int ti = 0; ti < NLM; ++ti)
#pragma unroll
        for (int tj = 0; tj < NLN; ++tj) {
          if (n0 + lcol + tj * MT >= g.N) continue;
          const float bias = g.aux[n0 + lcol + tj * MT];
#pragma unroll
          for (int r = 0; r < MM::kRegs; ++r) {
            const float v = fmaxf(acc[ti][tj][r] + bias, 0.0f);
            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), rc, voc,
                                                  (ti * MT + MM::row_reg(r)) * ldc4 + tj * MT * 4, 0);
          }
        }
    } else if (EPI == EPI_PARTIAL) {
#pragma unroll
      for (int ti = 0; ti < NLM; ++ti)
#pragma unroll
        for (int tj = 0; tj < NLN; ++tj) {
          if (n0 + lcol + tj * MT >= g.N) continue;
#pragma unroll
          for (int r = 0; r < MM::kRegs; ++r)
            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(acc[ti][tj][r]), rc, voc,
                                                  (ti * MT + MM::row_reg(r)) * ldc4 + tj * MT * 4, 0);
        }
    } else if (EPI == EPI_GRAD) {
      const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
          const_cast<float*>(g.aux) + (int64_t)m0 * g.ldaux + n0, 0, 0xffffffff, 0x00020000);
      const __amdgpu_buffer_rsrc_t rh = __builtin_amdgcn_make_buffer_rsrc(
          const_cast<float*>(Hq) + (int64_t)m0 * g.ldc + n0, 0, 0xffffffff, 0x00020000);
      const int vow = (lrow * (int)g.ldaux + lcol) * 4;
      const int lda4 = (int)g.ldaux * 4;
#pragma unroll
      for (int ti = 0; ti < NLM; ++ti)
#pragma unroll
        for (int tj = 0; tj < NLN; ++tj) {
          if (n0 + lcol + tj * MT >= g.N) continue;
          float wv[MM::kRegs], hv[MM::kRegs];
#pragma unroll
          for (int r = 0; r < MM::kRegs; ++r) {
            wv[r] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(
                rw, vow, (ti * MT + MM::row_reg(r)) * lda4 + tj * MT * 4, 0));
            hv[r] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(
                rh, voc, (ti * MT + MM::row_reg(r)) * ldc4 + tj * MT * 4, 0));
          }
#pragma unroll
          for (int r = 0; r < MM::kRegs; ++r) {
            const float v = fmaf(acc[ti][tj][r], g.scale, g.reg * wv[r]);
            const uint32_t db = __float_as_uint(v - hv[r]) & 0x7fffffffu;
            dmax = dmax > db ? dmax : db;
            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), rc, voc,
                                                  (ti * MT + MM::row_reg(r)) * ldc4 + tj * MT * 4, 0);
          }
        }
    } else {
      const __amdgpu_buffer_rsrc_t rm = __builtin_amdgcn_make_buffer_rsrc(
          const_cast<float*>(mask) + (int64_t)m0 * g.ldaux + n0, 0, 0xffffffff, 0x00020000);
      const int vom = (lrow * (int)g.ldaux + lcol) * 4;
      const int lda4 = (int)g.ldaux * 4;
#pragma unroll
      for (int ti = 0; ti < NLM; ++ti)
#pragma unroll
        for (int tj = 0; tj < NLN; ++tj) {
          if (n0 + lcol + tj * MT >= g.N) continue;
          float mk[MM::kRegs];
#pragma unroll
          for (int r = 0; r < MM::kRegs; ++r)
            mk[r] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(
                rm, vom, (ti * MT + MM::row_reg(r)) * lda4 + tj * MT * 4, 0));
#pragma unroll
          for (int r = 0; r < MM::kRegs; ++r) {
            const float v = mk[r] > 0.0f ? acc[ti][tj][r] : 0.0f;
            csum[tj] += v;
            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), rc, voc,
                                                  (ti * MT + MM::row_reg(r)) * ldc4 + tj * MT * 4, 0);
          }
        }
    }
  } else
#pragma unroll
  for (int ti = 0; ti < NLM; ++ti)
#pragma unroll
    for (int tj = 0; tj < NLN; ++tj) {
      const int col = n0 + (wx * NLN + tj) * MT + li;
      if (col >= g.N) continue;
      float bias = 0.0f;
      if (EPI == EPI_BIAS_RELU) bias = g.aux[col];
#pragma unroll
      for (int r = 0; r < MM::kRegs; ++r) {
        const int row = m0 + (wy * NLM + ti) * MT + MM::row(r, kh);
        if (row >= g.M) continue;
        float v = acc[ti][tj][r];
        if (EPI == EPI_BIAS_RELU) {
          v = fmaxf(v + bias, 0.0f);
        } else if (EPI == EPI_MASK) {
          v = mask[(int64_t)row * g.ldaux + col] > 0.0f ? v : 0.0f;
          csum[tj] += v;
        } else if (EPI == EPI_PARTIAL) {
          // plain product of this K range; scale, regulariser and radius follow in the slab sum
        } else {
          v = fmaf(v, g.scale, g.reg * g.aux[(int64_t)row * g.ldaux + col]);
          const uint32_t db = __float_as_uint(v - Hq[(int64_t)row * g.ldc + col]) & 0x7fffffffu;
          dmax = dmax > db ? dmax : db;
        }
        C[(int64_t)row * g.ldc + col] = v;
      }
    }
  if (EPI == EPI_MASK) {
    // column sums over the block's rows, in a fixed order: the lane's rows above, the tile's other rows
    // (the other k groups: lane ^ 32, and lane ^ 16 for 16 x 16 tiles), then the WM wavefront rows through
    // LDS (the A tile's, free since the K loop's last barrier)
    float* red = &As[0][0][0];
#pragma unroll
    for (int tj = 0; tj < NLN; ++tj) {
      float s = csum[tj] + __shfl_xor(csum[tj], 32);
      if (MT == 16) s += __shfl_xor(s, 16);
      if (kh == 0) red[wy * kBN + (wx * NLN + tj) * MT + li] = s;
    }
    __syncthreads();
    for (int c = threadIdx.x; c < kBN; c += kThreads) {
      if (n0 + c >= g.N) break;
      float s = red[c];
#pragma unroll
      for (int w = 1; w < WM; ++w) s += red[w * kBN + c];
      g.colpart[((int64_t)blockIdx.z * gridDim.y + blockIdx.y) * g.N + n0 + c] = s;
    }
  }
  if (EPI == EPI_GRAD) {
    // block maximum of |g - h| for the quantizer's radius (reuses the A tile's LDS)
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      const uint32_t o = (uint32_t)__shfl_xor((int)dmax, off);
      dmax = dmax > o ? dmax : o;
    }
    uint32_t* red = reinterpret_cast<uint32_t*>(&As[0][0][0]);
    if (lane == 0) red[wave] = dmax;
    __syncthreads();
    if (threadIdx.x == 0)
      g.rprod[(int64_t)blockIdx.z * g.rstride + g.rbase + g.slot0 + blockIdx.y * gridDim.x + blockIdx.x] =
          max(max(red[0], red[1]), max(red[2], red[3]));
  }
}

// Square block tiles of 64 NL: 2 x 2 wavefronts.  Four wavefronts per SIMD: 64 accumulator
// registers + at most 64 others.
template <bool TA, int EPI, int NL, bool FAST, bool RAGGED = false>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(4, 4))) void gemm_kernel(GemmArgs g) {
  gemm_body<TA, EPI, 2, NL, NL, FAST, RAGGED>(g);
}

// Layers between 129 and 224 units wide: one block tile spans the whole width (a 128 x 128 tiling would
// spend a second, mostly empty tile column on it), on 16 x 16 x 4 matrix instructions: block tile
// 64 x 16 NLN, each wavefront 16 rows by all NLN column tiles (4 NLN accumulator registers, four
// wavefronts per SIMD); the width pads to a multiple of 16 (200 -> 208) and 784 rows to 832.  (The same
// layers on 128 x 32 NLN tiles of 32 x 32 x 2 instructions, 112 accumulators and two wavefronts per SIMD,
// were 13 % slower: half as many blocks, 224 columns for 200, 896 rows for 784.)
template <bool TA, int EPI, int NLN, bool FAST>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(4, 4))) void gemm_narrow_kernel(GemmArgs g) {
  gemm_body<TA, EPI, 4, 1, NLN, FAST, false, 16>(g);
}

// ------------------------------------------------------------------ class layer (C <= 16)

constexpr int kCMax = 16;

// Class layer forward + loss gradient: Z[16 rows][C] = A[16][K] W[K][C] + b on
// v_mfma_f32_16x16x4_f32 (classes padded to 16), P = softmax(Z), dZ = P - onehot(y).
// A wavefront owns tiles of 16 rows and works alone: lane (row i = lane%16,
// quarter q = lane/16) streams A[i][16t + 4q .. +3] straight from HBM (each
// activation is used once) while W^T sits in LDS as the B operand; the softmax
// is a 16-lane butterfly on the accumulator layout.  No barrier in the loop.
// The kernel lives on loads in flight: four chunks (64 bytes per lane) are requested before the
// first is multiplied, and when W^T is so large that only one block fits a CU the block has
// sixteen wavefronts instead of four.
__global__ __launch_bounds__(1024) void class_forward_kernel(const float* __restrict__ Aact, int64_t lda,
                                                                 const float* __restrict__ W,
                                                                 const float* __restrict__ bias,
                                                                 const int32_t* __restrict__ y, int64_t S,
                                                                 int32_t K, int32_t C, int32_t ldsK, int32_t vec,
                                                                 float* __restrict__ dZ) {
  extern __shared__ __attribute__((aligned(16))) float Wt[];   // [C][ldsK], columns >= K zero
  const int nchunk = (K + 15) / 16, KP = nchunk * 16;
  // W^T into LDS, eight loads in flight per thread (unconditional, from clamped indices)
  for (int i0 = threadIdx.x; i0 < C * KP; i0 += 8 * (int)blockDim.x) {
    float wv[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int idx = i0 + u * (int)blockDim.x;
      const int c = idx / KP, k = idx - c * KP;
      wv[u] = W[(c < C && k < K) ? (int64_t)k * C + c : 0];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int idx = i0 + u * (int)blockDim.x;
      const int c = idx / KP, k = idx - c * KP;
      if (idx < C * KP) Wt[c * ldsK + k] = k < K ? wv[u] : 0.0f;
    }
  }
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l16 = lane & 15, lq = lane >> 4;
  const int64_t n_tiles = (S + 15) / 16;
  const int waves = (int)blockDim.x / 64;
  const int64_t stride = (int64_t)gridDim.x * waves;
  const float bj = l16 < C ? bias[l16] : 0.0f;
  for (int64_t tile = (int64_t)blockIdx.x * waves + wave; tile < n_tiles; tile += stride) {
    const int64_t row0 = tile * 16;
    int64_t ra = row0 + l16;
    ra = ra < S ? ra : S - 1;
    const float* arow = Aact + ra * lda + 4 * lq;
    const float* wrow = Wt + l16 * ldsK + 4 * lq;
    int ylab[4];                                      // labels of this lane's four rows, requested now
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int64_t row = row0 + 4 * lq + r;
      ylab[r] = y[row < S ? row : S - 1];
    }
    floatx4 acc0 = floatx4{0.f, 0.f, 0.f, 0.f}, acc1 = floatx4{0.f, 0.f, 0.f, 0.f};
    auto fetch = [&](int t) {
      const int k = 16 * t + 4 * lq;
      float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
      if (vec && k + 3 < K) {
        a = *reinterpret_cast<const float4*>(arow + 16 * t);
      } else {
        if (k < K) a.x = arow[16 * t];
        if (k + 1 < K) a.y = arow[16 * t + 1];
        if (k + 2 < K) a.z = arow[16 * t + 2];
        if (k + 3 < K) a.w = arow[16 * t + 3];
      }
      return a;
    };
    auto multiply = [&](int t, const float4& a, floatx4& acc) {
      float4 b = make_float4(0.f, 0.f, 0.f, 0.f);
      if (l16 < C) b = *reinterpret_cast<const float4*>(wrow + 16 * t);
      acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.x, b.x, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.y, b.y, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.z, b.z, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.w, b.w, acc, 0, 0, 0);
    };
    if (vec && (K & 3) == 0) {
      // aligned rows: eight unconditional loads in flight (chunks past the row repeat its last
      // float4, unused), nothing looks at a value before its turn to be multiplied
      for (int t0 = 0; t0 < nchunk; t0 += 8) {
        float4 a[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int k = 16 * (t0 + u) + 4 * lq;
          a[u] = *reinterpret_cast<const float4*>(arow - 4 * lq + (k < K ? k : K - 4));
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          if (t0 + u < nchunk) {                      // uniform
            const int k = 16 * (t0 + u) + 4 * lq;
            float4 v = a[u];
            if (k >= K) v = make_float4(0.f, 0.f, 0.f, 0.f);
            multiply(t0 + u, v, (u & 1) ? acc1 : acc0);
          }
        }
      }
    } else {
      int t = 0;
      for (; t + 3 < nchunk; t += 4) {   // four loads in flight, two independent accumulator chains
        const float4 a0 = fetch(t), a1 = fetch(t + 1), a2 = fetch(t + 2), a3 = fetch(t + 3);
        multiply(t, a0, acc0);
        multiply(t + 1, a1, acc1);
        multiply(t + 2, a2, acc0);
        multiply(t + 3, a3, acc1);
      }
      for (; t < nchunk; ++t) multiply(t, fetch(t), acc0);
    }
    // lane holds Z[4 lq + r][l16], r = 0..3
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int64_t row = row0 + 4 * lq + r;
      const bool valid = l16 < C;
      const float z = acc0[r] + acc1[r] + bj;
      float zm = valid ? z : -INFINITY;
#pragma unroll
      for (int off = 8; off > 0; off >>= 1) zm = fmaxf(zm, __shfl_xor(zm, off));
      const float e = valid ? expf(z - zm) : 0.0f;
      float den = e;
#pragma unroll
      for (int off = 8; off > 0; off >>= 1) den += __shfl_xor(den, off);
      if (valid && row < S) dZ[row * C + l16] = e / den - (l16 == ylab[r] ? 1.0f : 0.0f);
    }
  }
}

// Everything the class layer's residuals dZ[n][c] produce, for worker m and row slab blockIdx.y, in
// one pass over the activations A[n][i] of the last hidden layer (K units wide; the inputs if the
// network has no hidden layer):
//   weight gradient   part[..][kb + i C + c] = sum_{n in slab} A[n][i] dZ[n][c]
//   class bias        part[..][kb + K C + c] = sum_{n in slab} dZ[n][c]
// and, if a hidden layer precedes (has_prev; then kb = K, else kb = 0),
//   dZ_prev[n][i] = (A[n][i] > 0) ? sum_c dZ[n][c] W[i][c] : 0   and   part[..][i] = sum_{n in slab} dZ_prev[n][i]
// (the hidden layer's bias gradient).  The three partials sit in parameter order (b_{L-1}, W_L, b_L),
// so one slab sum finishes that whole stretch of the gradient.  A thread owns unit i; the residual
// rows of a chunk are staged in LDS (every lane reads the same row: broadcast reads) and eight rows
// of activations are in flight per step: the activations are streamed once, so the loop lives on
// memory latency.
__global__ __launch_bounds__(kThreads) void class_grads_kernel(const float* __restrict__ Aact, int64_t lda,
                                                               const float* __restrict__ dZ,
                                                               const float* __restrict__ W, int64_t N_m,
                                                               int32_t K, int32_t C, int32_t rows_per_slab,
                                                               int32_t has_prev, float* __restrict__ dZprev,
                                                               int64_t ldo, float* __restrict__ part,
                                                               int64_t part_stride) {
  const int m = blockIdx.z, slab = blockIdx.y;
  const int i = blockIdx.x * kThreads + threadIdx.x;
  const bool mine = i < K;
  const int64_t r0 = (int64_t)m * N_m + (int64_t)slab * rows_per_slab;
  int64_t r1 = r0 + rows_per_slab;
  const int64_t rend = (int64_t)(m + 1) * N_m;
  if (r1 > rend) r1 = rend;
  float acc[kCMax], w[kCMax];
#pragma unroll
  for (int c = 0; c < kCMax; ++c) {
    acc[c] = 0.0f;
    w[c] = (has_prev && mine && c < C) ? W[(int64_t)i * C + c] : 0.0f;
  }
  float bprev = 0.0f, bclass = 0.0f;
  const bool sums_class = blockIdx.x == 0 && (int)threadIdx.x < C;
  constexpr int kChunk = 128, kFly = 8;
  __shared__ __attribute__((aligned(16))) float dzs[kChunk][kCMax];
  const int64_t icl = mine ? i : 0;                     // idle lanes read column 0 and store nothing
  // rows n .. n+7 of the activations, always fetched (rows past the slab repeat its last row, unused):
  // a fetch under a branch would make the compiler wait for it on the spot
  auto fetch = [&](int64_t n, float (&v)[kFly]) {
#pragma unroll
    for (int u = 0; u < kFly; ++u) {
      const int64_t row = n + u < r1 ? n + u : r1 - 1;
      v[u] = Aact[row * lda + icl];
    }
  };
  float av[kFly], nx[kFly];
  if (r0 < r1) fetch(r0, av);
  for (int64_t n = r0; n < r1; n += kFly) {
    const int rr0 = (int)((n - r0) % kChunk);
    if (rr0 == 0) {                                     // next chunk of residual rows
      const int rows = (int)(r1 - n < kChunk ? r1 - n : kChunk);
      __syncthreads();
      for (int idx = threadIdx.x; idx < kChunk * kCMax; idx += kThreads) {
        const int rr = idx / kCMax, c = idx - rr * kCMax;
        dzs[rr][c] = (rr < rows && c < C) ? dZ[(n + rr) * C + c] : 0.0f;
      }
      __syncthreads();
      if (sums_class)
        for (int rr = 0; rr < rows; ++rr) bclass += dzs[rr][threadIdx.x];
    }
    fetch(n + kFly, nx);                                // the next group, while this one is used
#pragma unroll
    for (int u = 0; u < kFly; ++u) {
      if (n + u >= r1) break;
      const float a = av[u];
      const int rr = rr0 + u;
      float sacc = 0.0f;
#pragma unroll
      for (int c4 = 0; c4 < kCMax; c4 += 4) {
        if (c4 < C) {
          const float4 d = *reinterpret_cast<const float4*>(&dzs[rr][c4]);
          acc[c4] = fmaf(a, d.x, acc[c4]);
          acc[c4 + 1] = fmaf(a, d.y, acc[c4 + 1]);
          acc[c4 + 2] = fmaf(a, d.z, acc[c4 + 2]);
          acc[c4 + 3] = fmaf(a, d.w, acc[c4 + 3]);
          sacc = fmaf(d.x, w[c4], sacc);
          sacc = fmaf(d.y, w[c4 + 1], sacc);
          sacc = fmaf(d.z, w[c4 + 2], sacc);
          sacc = fmaf(d.w, w[c4 + 3], sacc);
        }
      }
      if (has_prev) {
        const float o = a > 0.0f ? sacc : 0.0f;
        if (mine) dZprev[(n + u) * ldo + i] = o;
        bprev += o;
      }
    }
#pragma unroll
    for (int u = 0; u < kFly; ++u) av[u] = nx[u];
  }
  float* out = part + ((int64_t)m * gridDim.y + slab) * part_stride;
  const int64_t kb = has_prev ? K : 0;
  if (mine) {
    if (has_prev) out[i] = bprev;
#pragma unroll
    for (int c = 0; c < kCMax; ++c)
      if (c < C) out[kb + (int64_t)i * C + c] = acc[c];
  }
  if (sums_class) out[kb + (int64_t)K * C + threadIdx.x] = bclass;
}

// Wt[c][r] = W[r][c] for W of R x Cn floats (rows packed): 32 x 32 tiles through LDS, both sides coalesced.
__global__ __launch_bounds__(kThreads) void transpose_kernel(const float* __restrict__ W, int32_t Rn, int32_t Cn,
                                                             float* __restrict__ Wt) {
  __shared__ float tile[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;          // 32 x 8
  const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
#pragma unroll
  for (int i = 0; i < 32; i += 8) {
    const int r = r0 + ty + i, c = c0 + tx;
    if (r < Rn && c < Cn) tile[ty + i][tx] = W[(int64_t)r * Cn + c];
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 32; i += 8) {
    const int c = c0 + ty + i, r = r0 + tx;
    if (r < Rn && c < Cn) Wt[(int64_t)c * Rn + r] = tile[tx][ty + i];
  }
}

// G[m][off + j] = (sum over slabs, ascending) part[m][slab][j] * scale + reg * theta[off + j],
// part rows `stride` floats apart.
// Also leaves the block maximum of |G - H| (raw bits) in rprod[m * rstride + rbase + blockIdx.x].
__global__ __launch_bounds__(kThreads) void slab_finish_kernel(const float* __restrict__ part, int32_t n_slab,
                                                               int64_t len, int64_t stride,
                                                               const float* __restrict__ theta_seg,
                                                               float scale, float reg, float* __restrict__ G,
                                                               const float* __restrict__ Hq, int64_t p_stride,
                                                               uint32_t* __restrict__ rprod, int32_t rstride,
                                                               int32_t rbase) {
  const int m = blockIdx.y;
  const int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  uint32_t mx = 0;
  if (j < len) {
    const float* pm = part + (int64_t)m * n_slab * stride;
    float s = 0.0f;
    // sixteen partials in flight (slabs past the last repeat it, unused), added in ascending order:
    // one memory latency per sixteen, not per one
    for (int k = 0; k < n_slab; k += 16) {
      float v[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const int ks = k + u < n_slab ? k + u : n_slab - 1;
        v[u] = pm[(int64_t)ks * stride + j];
      }
#pragma unroll
      for (int u = 0; u < 16; ++u)
        if (k + u < n_slab) s += v[u];
    }
    const float gv = fmaf(s, scale, reg * theta_seg[j]);
    G[(int64_t)m * p_stride + j] = gv;
    mx = __float_as_uint(gv - Hq[(int64_t)m * p_stride + j]) & 0x7fffffffu;
  }
  __shared__ uint32_t sm[kThreads / 64];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const uint32_t o = (uint32_t)__shfl_xor((int)mx, off);
    mx = mx > o ? mx : o;
  }
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = mx;
  __syncthreads();
  if (threadIdx.x == 0)
    rprod[(int64_t)m * rstride + rbase + blockIdx.x] = max(max(sm[0], sm[1]), max(sm[2], sm[3]));
}

// ------------------------------------------------------------------ host side

static inline int64_t align_up(int64_t a, int64_t b) { return (a + b - 1) / b * b; }

struct GemmTile { int bm, bn; int mt = 32; };   // block tile and the matrix-instruction tile it is made of

// Block tile: 128 x 128 when that still gives every CU a few blocks, else 64 x 64; 64 x (160, 192, 208
// or 224) of 16 x 16 matrix tiles for an output 129..224 columns wide with enough rows of tiles to occupy
// the chip.
// big: the caller fills the chip by other means (split K) and wants the large tiles.
static GemmTile gemm_tile(const laq_ctx* ctx, int64_t Mr, int64_t Nc, int batch, bool big = false) {
  if (Nc > 128 && Nc <= 224 && (big || ((Mr + 63) / 64) * batch >= (int64_t)ctx->n_cu)) {
    const int w = Nc <= 160 ? 160 : (Nc <= 192 ? 192 : (Nc <= 208 ? 208 : 224));
    return GemmTile{64, w, 16};
  }
  const int64_t blocks128 = ((Mr + 127) / 128) * ((Nc + 127) / 128) * batch;
  const int bt = (big || blocks128 >= (int64_t)ctx->n_cu * 3) ? 128 : 64;
  return GemmTile{bt, bt};
}

// Rows of a per-worker weight gradient past its last full row of 128 x 128 tiles, when they are launched
// on their own: at most 64 of them (784 rows: 16), in 64 x 64 tiles whose empty 32-row halves take no matrix
// instructions.  As a seventh row of 128 x 128 tiles they would cost a seventh of the product.
static int ragged_rows(GemmTile t, int64_t Mr) {
  const int rem = (int)(Mr % 128);
  return (t.bm == 128 && t.bn == 128 && rem != 0 && rem <= 64) ? rem : 0;
}
// Blocks (= radius slots) of a weight-gradient launch of Mr x Nc outputs per worker
static int64_t dw_blocks(GemmTile t, int64_t Mr, int64_t Nc) {
  if (ragged_rows(t, Mr)) return (Mr / 128) * ((Nc + 127) / 128) + (Nc + 63) / 64;
  return ((Mr + t.bm - 1) / t.bm) * ((Nc + t.bn - 1) / t.bn);
}

// Weight-gradient GEMMs whose large tiles would leave most CUs idle (narrow layers) split the
// sample dimension: nsplit partial products per worker, summed by slab_finish_kernel.  All blocks
// of such a launch are resident at once or nearly so, so the launch takes as long as the
// fullest CU: nsplit is the value whose block count fills whole rounds of CUs best.
static int dw_splits(const laq_ctx* ctx, int64_t in, int64_t out, int64_t N_m) {
  const GemmTile t = gemm_tile(ctx, in, out, ctx->M, true);
  const int64_t blocks1 = ((in + t.bm - 1) / t.bm) * ((out + t.bn - 1) / t.bn) * ctx->M;
  if (blocks1 >= (int64_t)ctx->n_cu * 3) return 1;
  int64_t max_ns = N_m / 512;                  // at least 512 samples per split
  if (max_ns > 16) max_ns = 16;
  int best = 1;
  double best_fill = 0.0;
  for (int64_t ns = 2; ns <= max_ns; ++ns) {
    const int64_t blocks = blocks1 * ns;
    if (blocks > (int64_t)ctx->n_cu * 4) break;
    const int64_t rounds = (blocks + ctx->n_cu - 1) / ctx->n_cu;
    const double fill = (double)blocks / (double)(rounds * ctx->n_cu);
    if (fill > best_fill + 0.02) { best_fill = fill; best = (int)ns; }   // near-ties: fewer partials
  }
  return best;
}

struct MlpPlan {
  int64_t S;
  int64_t act_off[LAQ_MAX_LAYERS];   // activations after hidden layer l (l = 1..L-1), floats
  int64_t dz_off[LAQ_MAX_LAYERS];    // gradients w.r.t. pre-activations of hidden layer l
  int64_t dzc_off;                   // [S][C]
  int64_t part_off;                  // slab partial sums
  int64_t part_len;                  // floats per (worker, slab)
  int32_t n_slab, rows_per_slab;
  int64_t rprod_off;                 // [M][rprod_count] block maxima of |g - h|
  int32_t rprod_count;
  int64_t splitk_off;                // [M][nsplit][in * out] partial weight gradients (largest split layer)
  int64_t wt_off;                    // transposed copy of the weights an activation-gradient product reads
  int64_t total_floats;
};

static MlpPlan make_plan(const laq_ctx* ctx, int64_t N_m) {
  const Mlp& n = ctx->mlp;
  MlpPlan pl{};
  pl.S = (int64_t)ctx->M * N_m;
  int64_t off = 0;
  for (int l = 1; l < n.n_layers; ++l) {
    pl.act_off[l] = off; off += align_up(pl.S * n.dims[l], 64);
    pl.dz_off[l] = off; off += align_up(pl.S * n.dims[l], 64);
  }
  pl.dzc_off = off; off += align_up(pl.S * n.dims[n.n_layers], 64);
  // slabs of rows for the bandwidth-bound reductions (class-layer weights, biases)
  int64_t want = ((int64_t)ctx->n_cu * 6 + ctx->M - 1) / ctx->M;
  if (want < 1) want = 1;
  int64_t rps = (N_m + want - 1) / want;
  if (rps < 32) rps = 32;
  if (rps > N_m) rps = N_m;
  pl.rows_per_slab = (int32_t)rps;
  pl.n_slab = (int32_t)((N_m + rps - 1) / rps);
  int64_t widest = 0;
  for (int l = 1; l <= n.n_layers; ++l) widest = widest > n.dims[l] ? widest : n.dims[l];
  // class_grads_kernel leaves (b_{L-1} |) W_L | b_L partials side by side
  const int64_t Kc = n.dims[n.n_layers - 1], Cc = n.dims[n.n_layers];
  const int64_t class_len = (n.n_layers >= 2 ? Kc : 0) + Kc * Cc + Cc;
  const int64_t part_len = class_len > widest ? class_len : widest;
  pl.part_len = part_len;
  // the same buffer takes the bias-gradient partials of the earlier hidden layers: one row of sums per row
  // of block tiles of the activation-gradient product
  int64_t part_floats = (int64_t)ctx->M * pl.n_slab * part_len;
  for (int l = 1; l < n.n_layers - 1; ++l) {
    const GemmTile t = gemm_tile(ctx, N_m, n.dims[l], ctx->M);
    const int64_t need = (int64_t)ctx->M * ((N_m + t.bm - 1) / t.bm) * n.dims[l];
    part_floats = part_floats > need ? part_floats : need;
  }
  pl.part_off = off; off += align_up(part_floats, 64);
  // one radius slot per block of every kernel that writes a segment of G
  int64_t cnt = 0, splitk = 0;
  for (int l = 1; l <= n.n_layers; ++l) {
    const int64_t in = n.dims[l - 1], out = n.dims[l];
    if (l < n.n_layers) {                                                         // weight-gradient GEMM
      const int ns = dw_splits(ctx, in, out, N_m);
      if (ns > 1) {
        cnt += (in * out + kThreads - 1) / kThreads;                                // summed by slab_finish_kernel
        const int64_t need = (int64_t)ctx->M * ns * in * out;
        splitk = splitk > need ? splitk : need;
      } else {
        cnt += dw_blocks(gemm_tile(ctx, in, out, ctx->M), in, out);
      }
    }
    else cnt += (class_len + kThreads - 1) / kThreads;     // class layer, its bias, the last hidden layer's bias
    if (l < n.n_layers - 1) cnt += (out + kThreads - 1) / kThreads;                 // bias of an earlier hidden layer
  }
  pl.rprod_count = (int32_t)cnt;
  pl.rprod_off = off; off += align_up((int64_t)ctx->M * cnt, 64);
  pl.splitk_off = off; off += align_up(splitk, 64);
  int64_t wt = 0;
  for (int l = 1; l < n.n_layers - 1; ++l) {
    const int64_t need = (int64_t)n.dims[l] * n.dims[l + 1];
    wt = wt > need ? wt : need;
  }
  pl.wt_off = off; off += align_up(wt, 64);
  pl.total_floats = off;
  return pl;
}

size_t mlp_workspace_bytes(const laq_ctx* ctx, int64_t N_m) {
  return (size_t)make_plan(ctx, N_m).total_floats * sizeof(float) + 256;
}

static size_t gemm_lds_bytes(GemmTile t, bool ta) {
  const int lda = !ta ? t.bm : (t.mt == 32 ? lds_stride<32>(t.bm) : lds_stride<16>(t.bm));
  const int ldb = t.mt == 32 ? lds_stride<32>(t.bn) : lds_stride<16>(t.bn);
  return (size_t)LAQ_GEMM_NBUF * LAQ_GEMM_BK * (lda + ldb) * sizeof(float);
}

template <bool TA, int EPI>
static void launch_gemm(const laq_ctx* ctx, const GemmArgs& g, int batch, bool big = false) {
  const GemmTile t = gemm_tile(ctx, g.M, g.N, batch, big);
  const dim3 grid((unsigned)((g.N + t.bn - 1) / t.bn), (unsigned)((g.M + t.bm - 1) / t.bm), (unsigned)batch);
  // fast loaders need aligned operand rows and no float4 straddling an operand edge
  // ... and row strides whose tile offsets fit the loaders' 32-bit lane offsets
  const bool fast = g.vecA && g.vecB && (g.M % 4 == 0) && (g.N % 4 == 0) && (g.K % 4 == 0) && g.K >= 4 &&
                    g.lda <= ((int64_t)1 << 30) / 224 - 64 && g.ldb <= ((int64_t)1 << 30) / 224 - 64;
  const size_t smem = gemm_lds_bytes(t, TA);
#define LAQ_GEMM_LAUNCH(KERNEL, P)                                                                            \
  do {                                                                                                        \
    if (fast) hipLaunchKernelGGL((KERNEL<TA, EPI, P, true>), grid, dim3(kThreads), smem, ctx->stream, g);  \
    else hipLaunchKernelGGL((KERNEL<TA, EPI, P, false>), grid, dim3(kThreads), smem, ctx->stream, g);      \
  } while (0)
  if (t.mt == 16) {
    if (t.bn == 160) LAQ_GEMM_LAUNCH(gemm_narrow_kernel, 10);
    else if (t.bn == 192) LAQ_GEMM_LAUNCH(gemm_narrow_kernel, 12);
    else if (t.bn == 208) LAQ_GEMM_LAUNCH(gemm_narrow_kernel, 13);
    else LAQ_GEMM_LAUNCH(gemm_narrow_kernel, 14);
  } else if (t.bn == t.bm) {
    if (t.bm == 128) {
      // per-worker weight gradients: the rows past the last full row of tiles go in a launch of their own
      if constexpr (TA) if (ragged_rows(t, g.M)) {
        const int full = g.M / 128;
        if (full > 0) {
          const dim3 gi(grid.x, (unsigned)full, grid.z);
          if (fast) hipLaunchKernelGGL((gemm_kernel<TA, EPI, 2, true>), gi, dim3(kThreads), smem, ctx->stream, g);
          else hipLaunchKernelGGL((gemm_kernel<TA, EPI, 2, false>), gi, dim3(kThreads), smem, ctx->stream, g);
        }
        GemmArgs ge = g;
        ge.y0 = 2 * full;                                   // in rows of 64 x 64 tiles
        ge.slot0 = full * (int32_t)grid.x;
        const dim3 gr((unsigned)((g.N + 63) / 64), 1, grid.z);
        const size_t smem_r = gemm_lds_bytes(GemmTile{64, 64}, TA);
        if (fast) hipLaunchKernelGGL((gemm_kernel<TA, EPI, 1, true, true>), gr, dim3(kThreads), smem_r, ctx->stream, ge);
        else hipLaunchKernelGGL((gemm_kernel<TA, EPI, 1, false, true>), gr, dim3(kThreads), smem_r, ctx->stream, ge);
        return;
      }
      LAQ_GEMM_LAUNCH(gemm_kernel, 2);
    }
    else LAQ_GEMM_LAUNCH(gemm_kernel, 1);
  }
#undef LAQ_GEMM_LAUNCH
}

static inline int vec_ok(const void* p, int64_t ld) { return (((uintptr_t)p & 15) == 0 && (ld & 3) == 0) ? 1 : 0; }

int mlp_worker_grads(laq_ctx* ctx, const float* theta, float* G) {
  const Mlp& n = ctx->mlp;
  const int L = n.n_layers;
  const int C = n.dims[L];
  if (C > kCMax) return set_error(ctx, LAQ_EINVAL, "MLP: at most %d classes (got %d)", kCMax, C);
  const int64_t N_m = ctx->N_m;
  const MlpPlan pl = make_plan(ctx, N_m);
  float* ws = reinterpret_cast<float*>(ctx->model_ws);
  const int64_t S = pl.S;
  const int64_t N = S;
  const float inv_N = (float)(1.0 / (double)N);
  const float reg = (float)(((double)N_m / (double)N) * (double)ctx->lambda);

  // ---- forward through the hidden layers: A_l = relu(A_{l-1} W_l + b_l)
  const float* Ain = ctx->X;
  int64_t ld_in = ctx->ldx;
  for (int l = 1; l < L; ++l) {
    GemmArgs g{};
    g.A = Ain; g.lda = ld_in;
    g.B = theta + n.offW[l - 1]; g.ldb = n.dims[l];
    g.C = ws + pl.act_off[l]; g.ldc = n.dims[l];
    g.M = (int32_t)S; g.N = n.dims[l]; g.K = n.dims[l - 1];
    g.vecA = vec_ok(g.A, g.lda); g.vecB = vec_ok(g.B, g.ldb);
    g.aux = theta + n.offB[l - 1];
    if (S > 0x7fffffff) return set_error(ctx, LAQ_EINVAL, "MLP: too many samples");
    launch_gemm<false, EPI_BIAS_RELU>(ctx, g, 1);
    Ain = g.C; ld_in = g.ldc;
  }
  // ---- class layer forward + softmax cross-entropy: dZ_L = P - Y
  float* dZc = ws + pl.dzc_off;
  {
    const int K = n.dims[L - 1];
    const int KP = (K + 15) / 16 * 16;
    const int ldsK = KP + (20 - KP % 32 + 32) % 32;   // row stride = 20 (mod 32) banks
    const size_t smem = (size_t)C * ldsK * sizeof(float);
    if (smem > 160 * 1024)
      return set_error(ctx, LAQ_EINVAL, "MLP: last hidden width * classes does not fit LDS");
    const int64_t tiles = (S + 15) / 16;
    const int cf_threads = smem > 40 * 1024 ? 1024 : kThreads;      // one block per CU: make it a large one
    const int cf_waves = cf_threads / 64;
    int64_t blocks = (tiles + cf_waves - 1) / cf_waves;
    const int64_t cap = (int64_t)ctx->n_cu * (cf_threads == kThreads ? 8 : 1);
    if (blocks > cap) blocks = cap;
    if (smem > 48 * 1024)
      LAQ_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(class_forward_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    hipLaunchKernelGGL(class_forward_kernel, dim3((unsigned)blocks), dim3((unsigned)cf_threads), smem, ctx->stream, Ain,
                       ld_in, theta + n.offW[L - 1], theta + n.offB[L - 1], ctx->y, S, K, C, ldsK,
                       vec_ok(Ain, ld_in), dZc);
  }
  float* part = ws + pl.part_off;
  // radius slots: every kernel that writes a segment of G gets its own range
  uint32_t* rprod = reinterpret_cast<uint32_t*>(ws + pl.rprod_off);
  const int32_t rstride = pl.rprod_count;
  int32_t rbase = 0;
  ctx->rprod = rprod; ctx->rprod_stride = rstride; ctx->rprod_count = pl.rprod_count;
  // ---- class layer gradients, the residuals of the last hidden layer and its bias gradient
  {
    const int K = n.dims[L - 1];
    const int has_prev = L >= 2 ? 1 : 0;
    if (has_prev && n.offB[L - 2] + K != n.offW[L - 1])
      return set_error(ctx, LAQ_EDEVICE, "internal: parameter layout is not (W_1, b_1, W_2, b_2, ...)");
    if (n.offW[L - 1] + (int64_t)K * C != n.offB[L - 1])
      return set_error(ctx, LAQ_EDEVICE, "internal: parameter layout is not (W_1, b_1, W_2, b_2, ...)");
    const int64_t len = (has_prev ? K : 0) + (int64_t)K * C + C;
    const int64_t seg = has_prev ? n.offB[L - 2] : n.offW[L - 1];
    float* dZprev = has_prev ? ws + pl.dz_off[L - 1] : nullptr;
    const dim3 wg((unsigned)((K + kThreads - 1) / kThreads), (unsigned)pl.n_slab, (unsigned)ctx->M);
    hipLaunchKernelGGL(class_grads_kernel, wg, dim3(kThreads), 0, ctx->stream, Ain, ld_in, dZc,
                       theta + n.offW[L - 1], N_m, K, C, pl.rows_per_slab, has_prev, dZprev, (int64_t)K, part,
                       pl.part_len);
    const unsigned wblocks = (unsigned)((len + kThreads - 1) / kThreads);
    hipLaunchKernelGGL(slab_finish_kernel, dim3(wblocks, (unsigned)ctx->M), dim3(kThreads), 0, ctx->stream, part,
                       pl.n_slab, len, pl.part_len, theta + seg, inv_N, reg, G + seg, ctx->H + seg, ctx->p_stride,
                       rprod, rstride, rbase);
    rbase += (int32_t)wblocks;
  }
  // ---- backward through the hidden layers
  const float* dZnext = dZc;     // gradient w.r.t. pre-activations of layer l+1
  for (int l = L - 1; l >= 1; --l) {
    float* dZl = ws + pl.dz_off[l];
    const float* Al = ws + pl.act_off[l];
    const int width = n.dims[l];
    if (l < L - 1) {            // (the class layer's kernel has already left dZ_{L-1})
      // dZ_l = (dZ_{l+1} W_{l+1}^T) .* (A_l > 0)
      // one batch entry per worker, so that no block tile holds rows of two workers: the epilogue also
      // leaves the column sums of its rows, the partial sums of db_l(m)
      // W_{l+1}[d_l][d_{l+1}] is this product's [N][K] operand; from a transposed copy [K][N] its tile loads
      // go to LDS as they are (16-byte stores), like the forward product's weights
      float* Wt = ws + pl.wt_off;
      hipLaunchKernelGGL(transpose_kernel, dim3((unsigned)((n.dims[l + 1] + 31) / 32), (unsigned)((width + 31) / 32)),
                         dim3(kThreads), 0, ctx->stream, theta + n.offW[l], width, n.dims[l + 1], Wt);
      GemmArgs g{};
      g.A = dZnext; g.lda = n.dims[l + 1]; g.sA = N_m * g.lda;
      g.B = Wt; g.ldb = width;
      g.C = dZl; g.ldc = width; g.sC = N_m * g.ldc;
      g.M = (int32_t)N_m; g.N = width; g.K = n.dims[l + 1];
      g.vecA = vec_ok(g.A, g.lda); g.vecB = vec_ok(g.B, g.ldb);
      g.aux = Al; g.ldaux = width; g.saux = N_m * g.ldaux;
      g.colpart = part;
      launch_gemm<false, EPI_MASK>(ctx, g, ctx->M);
      // db_l(m) = sum of those partials, scaled, + regulariser
      const GemmTile t = gemm_tile(ctx, N_m, width, ctx->M);
      const int32_t n_rowtiles = (int32_t)((N_m + t.bm - 1) / t.bm);
      const unsigned bblocks = (unsigned)((width + kThreads - 1) / kThreads);
      hipLaunchKernelGGL(slab_finish_kernel, dim3(bblocks, (unsigned)ctx->M), dim3(kThreads), 0, ctx->stream,
                         part, n_rowtiles, (int64_t)width, (int64_t)width, theta + n.offB[l - 1], inv_N, reg,
                         G + n.offB[l - 1], ctx->H + n.offB[l - 1], ctx->p_stride, rprod, rstride, rbase);
      rbase += (int32_t)bblocks;
    }
    // dW_l(m) = A_{l-1}(m)^T dZ_l(m), scaled, + regulariser -> G[m][offW_{l-1}]
    {
      const float* Aprev = (l == 1) ? ctx->X : ws + pl.act_off[l - 1];
      const int64_t ldp = (l == 1) ? ctx->ldx : n.dims[l - 1];
      GemmArgs g{};
      g.A = Aprev; g.lda = ldp; g.sA = N_m * ldp;
      g.B = dZl; g.ldb = width; g.sB = N_m * (int64_t)width;
      g.C = G + n.offW[l - 1]; g.ldc = width; g.sC = ctx->p_stride;
      g.M = n.dims[l - 1]; g.N = width; g.K = (int32_t)N_m;
      g.vecA = vec_ok(g.A, g.lda) && ((g.sA & 3) == 0);
      g.vecB = vec_ok(g.B, g.ldb) && ((g.sB & 3) == 0);
      g.aux = theta + n.offW[l - 1]; g.ldaux = width;
      g.scale = inv_N; g.reg = reg;
      g.Hq = ctx->H + n.offW[l - 1]; g.rprod = rprod; g.rstride = rstride; g.rbase = rbase;
      const int ns = dw_splits(ctx, g.M, g.N, N_m);
      if (ns > 1) {
        const int64_t len = (int64_t)g.M * g.N;
        float* sp = ws + pl.splitk_off;
        g.C = sp; g.sC = len;
        g.nsplit = ns;
        g.ksplit = (int32_t)align_up((N_m + ns - 1) / ns, 16);
        launch_gemm<true, EPI_PARTIAL>(ctx, g, ctx->M * ns, true);
        const unsigned wblocks = (unsigned)((len + kThreads - 1) / kThreads);
        hipLaunchKernelGGL(slab_finish_kernel, dim3(wblocks, (unsigned)ctx->M), dim3(kThreads), 0, ctx->stream, sp,
                           ns, len, len, theta + n.offW[l - 1], inv_N, reg, G + n.offW[l - 1],
                           ctx->H + n.offW[l - 1], ctx->p_stride, rprod, rstride, rbase);
        rbase += (int32_t)wblocks;
      } else {
        launch_gemm<true, EPI_GRAD>(ctx, g, ctx->M);
        rbase += (int32_t)dw_blocks(gemm_tile(ctx, g.M, g.N, ctx->M), g.M, g.N);
      }
    }
    dZnext = dZl;
  }
  if (rbase != pl.rprod_count)
    return set_error(ctx, LAQ_EDEVICE, "internal: radius slot count mismatch (%d vs %d)", rbase, pl.rprod_count);
  LAQ_HIP(ctx, hipGetLastError());
  return LAQ_OK;
}

}  // namespace laq
