// Tile addressing of the matrix kernels (laq_mlp.hip), in a form that also compiles for the host: the
// kernels read operands with unconditional, clamped 16-byte loads, so that every address they form must
// lie inside the operand for every tile shape, contraction length and width.  A host program walks the same
// functions over all 256 lanes and all tiles and checks exactly that (tests/test_loader_addresses.py); the
// lane number is therefore an argument, not threadIdx.x.
#pragma once

#include <stdint.h>

#if defined(__HIPCC__)
#define LAQ_HD __host__ __device__ __forceinline__
#else
#define LAQ_HD inline
#endif

namespace laq {

constexpr int kLoaderThreads = 256;   // lanes that share one tile (block size of the matrix kernels)

// An operand's block tile is BX wide and BK deep, BX BK / 4 float4 in all: lane t moves the float4
// numbered e = t + 256 i, i < NV = ceil(BX BK / 1024); when BX BK is not a multiple of 1024 the last of
// them does not exist for some lanes.  LDS tiles are K-major: tile[kk][xx].
template <int BX, int BK>
struct TileMap {
  static constexpr int kVec = BX * BK / 4;                       // float4 per tile
  static constexpr int NV = (kVec + kLoaderThreads - 1) / kLoaderThreads;
  static constexpr bool kExact = (kVec % kLoaderThreads) == 0;
  static constexpr int TPR = BX / 4;                             // lanes per tile row (K-major source)
  static constexpr int LPR = BK / 4;                             // lanes per source row (X-major source)
  static LAQ_HD bool exists(int tid, int i) { return kExact || tid + kLoaderThreads * i < kVec; }
  // K-major source S[k][x]: float4 e covers tile[kk][xx .. xx+3]
  static LAQ_HD void kmajor(int tid, int i, int& kk, int& xx) {
    const int e = tid + kLoaderThreads * i;
    kk = e / TPR; xx = (e % TPR) * 4;
  }
  // X-major source S[x][k]: float4 e covers tile[kk .. kk+3][xx]
  static LAQ_HD void xmajor(int tid, int i, int& kk, int& xx) {
    const int e = tid + kLoaderThreads * i;
    xx = e / LPR; kk = (e % LPR) * 4;
  }
};

// Fast path (operand rows 16-byte aligned, X and K multiples of 4, K >= 4): every float4 is wholly inside
// or wholly outside the operand, so a lane loads unconditionally from a clamped place and zeroes what lies
// outside.  No branch sits between the loads and the matrix instructions they overlap, and no vector
// instruction computes an address inside the K loop: a lane's float4 lies at
//     tile origin (uniform: x = x0, k = 0)  +  tile number * kstep (uniform)  +  voff (per lane, constant),
// which the kernel feeds to a buffer load as a scalar base and a 32-bit lane offset.  This struct holds the
// addressing (offsets in floats from the operand's first element); the loads themselves are in the kernel.
template <int BX, int BK, bool XMAJOR>
struct FastLoaderAddr {
  using TM = TileMap<BX, BK>;
  static constexpr int NV = TM::NV;
  uint32_t voff[NV];    // BYTE offset of this lane's float4 of K tile 0 from the tile origin (clamped into the operand)
  int kk[NV];           // its k offset inside the tile
  bool xin[NV];         // its row/column lies inside the operand (false for a float4 that does not exist)
  int64_t origin;       // float offset of the tile origin from the operand's first element
  int64_t kstep;        // float offset advance per K tile
  int64_t kunit;        // float offset advance per unit of k
  int K;
  bool all_in;          // the whole block tile lies inside the operand (uniform over the block)

  // (Every byte offset the kernel forms -- voff plus one K tile's advance -- must fit 32 bits: the host takes
  // this path only for row strides up to 2^30 / 224 - 64 floats.)
  // Operand K-major S[k][x] (XMAJOR false) or X-major S[x][k]; ld: its row stride; the block tile starts at x0.
  LAQ_HD void init(int tid, int64_t ld, int K_, int X, int x0) {
    K = K_;
    all_in = TM::kExact && x0 + BX <= X;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      int kq, xx;
      if (XMAJOR) TM::xmajor(tid, i, kq, xx); else TM::kmajor(tid, i, kq, xx);
      if (!TM::exists(tid, i)) { kq = 0; xx = 0; }
      kk[i] = kq;
      xin[i] = TM::exists(tid, i) && x0 + xx < X;
      const int xr = xin[i] ? xx : 0;                  // a float4 outside the operand reads the tile's first row / column
      voff[i] = (uint32_t)(4 * (XMAJOR ? (int64_t)xr * ld + kq : (int64_t)kq * ld + xr));
    }
    origin = XMAJOR ? (int64_t)x0 * ld : (int64_t)x0;
    kstep = XMAJOR ? BK : (int64_t)BK * ld;
    kunit = XMAJOR ? 1 : ld;
  }
  LAQ_HD bool is_whole(int tile) const { return tile * BK + BK <= K; }
  // Whole K tile `tile`: base (uniform) and the lane's float4
  LAQ_HD int64_t base(int tile) const { return origin + (int64_t)tile * kstep; }
  LAQ_HD int64_t whole(int tile, int i) const { return base(tile) + (int64_t)(voff[i] >> 2); }
  // The last, partial tile.  A float4 of k >= K is redirected to a place that is inside the operand
  // whatever K: its own place one K tile earlier (a whole tile) when there is one, else (K < BK, the
  // first tile is itself the partial one) k = 0 .. 3 of its own row or column.  The kernel reads the
  // partial tile from the base of the tile before it (of tile 0 if there is none) with these lane offsets:
  LAQ_HD int64_t partial_base(int tile) const { return base(tile >= 1 ? tile - 1 : 0); }
  LAQ_HD uint32_t partial_voff(int tile, int i) const {
    const bool kin = tile * BK + kk[i] < K;
    if (tile >= 1) return kin ? voff[i] + (uint32_t)(4 * kstep) : voff[i];
    return kin ? voff[i] : voff[i] - (uint32_t)(4 * kk[i] * kunit);
  }
  LAQ_HD int64_t partial(int tile, int i) const { return partial_base(tile) + (int64_t)(partial_voff(tile, i) >> 2); }
  // whether float4 i of K tile `tile` holds operand data (else it is zeroed on the way to LDS)
  LAQ_HD bool keep(int tile, int i) const { return (tile * BK + kk[i] < K) && xin[i]; }
};

}  // namespace laq

// ------------------------------------------------------------------ softmax-regression kernel (laq_grads.hip)
//
// Addressing of the matrix-core softmax-regression kernel's tile loads, shared with the host for the
// same reason.  A block of 16 wavefronts walks tiles of 16 rows; lane (l16 = row, lq = quarter) of wave w
// takes 16 bytes of each chunk w + 16 n (16 columns) of its row.  Tiles the prologue requests past the
// block's row range are clamped to its last row, rows past a ragged last tile to the tile's last row,
// and a chunk that may cross column F is clamped into the row; what was clamped is zeroed when used.
namespace laq {

constexpr int kSmxRowsPerTile = 16;
constexpr int kSmxWavesPerBlock = 16;

// first row of the tile requested at r0, clamped into the block's range [.., r_end)
LAQ_HD int64_t smx_tile_row(int64_t r0, int64_t r_end) { return r0 < r_end ? r0 : r_end - 1; }
// rows of that tile inside the range
LAQ_HD int smx_rows_valid(int64_t rb, int64_t r_end) {
  return (int)(r_end - rb < kSmxRowsPerTile ? r_end - rb : kSmxRowsPerTile);
}
// row inside the tile whose data lane l16 loads / whose label the lane's softmax row needs
LAQ_HD int smx_data_row(int l16, int rows_valid) { return l16 < rows_valid ? l16 : rows_valid - 1; }
LAQ_HD int smx_label_row(int wave, int lq, int rows_valid) {
  const int yrow = 4 * (wave & 3) + lq;                         // softmax waves 0..3: rows 4 wave + lq
  return yrow < rows_valid ? yrow : rows_valid - 1;
}
// float offset inside a row of the lane's 16 bytes of chunk `wave`; chunk wave + 16 n lies
// smx_chunk_step(n) floats further when it is wholly inside the F columns
LAQ_HD uint32_t smx_lane_col(int wave, int lq) { return 4u * (4u * (uint32_t)wave + (uint32_t)lq); }
LAQ_HD uint32_t smx_chunk_step(int n) { return 16u * (uint32_t)kSmxWavesPerBlock * (uint32_t)n; }
// the same for a chunk that may cross column F: its float4 column, or column 0 if the row (nf4r float4
// long, padding included) ends before it
LAQ_HD uint32_t smx_ragged_col(int wave, int n, int lq, int nf4r) {
  uint32_t q = 4u * (uint32_t)(wave + kSmxWavesPerBlock * n) + (uint32_t)lq;
  q = q < (uint32_t)nf4r ? q : 0u;
  return 4u * q;
}
// tiled copy: byte offset, inside the worker's tiled shard, of chunk `wave` of the tile holding row rb
// (of chunk 0 for a wave past the tile's last chunk), and of chunk wave + 16 n (the wave's first chunk
// again if the tile has no such chunk); the lane adds its own 16 l bytes
LAQ_HD uint32_t smx_tiled_tile_off(int64_t rb, int nchunk, int wave) {
  return (uint32_t)(rb / kSmxRowsPerTile) * (uint32_t)(nchunk * 1024) + 1024u * (uint32_t)(wave < nchunk ? wave : 0);
}
LAQ_HD uint32_t smx_tiled_chunk_off(uint32_t tile_off, int n, int nfull, int wave, int nchunk) {
  return tile_off + ((n < nfull || wave + kSmxWavesPerBlock * n < nchunk) ? 1024u * (uint32_t)kSmxWavesPerBlock * (uint32_t)n : 0u);
}
// kernel instantiation for F columns: chunks per wave (TMAX) and how many of them exist for every wave and
// hold no column >= F (NFULL); the tiled copy is zero-padded, so all its chunks count as whole
LAQ_HD void smx_variant(int F, bool tiled, int& tmax, int& nfull) {
  const int nchunk = (F + 15) / 16;
  const int whole = (tiled ? nchunk : F / 16) / kSmxWavesPerBlock;
  if (nchunk <= kSmxWavesPerBlock) { tmax = 1; nfull = whole >= 1 ? 1 : 0; }
  else if (nchunk <= 2 * kSmxWavesPerBlock) { tmax = 2; nfull = whole >= 2 ? 2 : 1; }
  else { tmax = 4; nfull = whole >= 4 ? 4 : (whole == 3 ? 3 : 2); }
}
// rows per block and number of blocks per worker: one block per CU at most, whole tiles per block
LAQ_HD int smx_blocks(int n_cu, int M, int64_t N_m, int* rows_per_block) {
  int64_t want = n_cu / M;
  if (want < 1) want = 1;
  const int64_t tiles = (N_m + kSmxRowsPerTile - 1) / kSmxRowsPerTile;
  if (want > tiles) want = tiles;
  const int64_t tpb = (tiles + want - 1) / want;
  *rows_per_block = (int)(tpb * kSmxRowsPerTile);
  return (int)((tiles + tpb - 1) / tpb);
}

}  // namespace laq
