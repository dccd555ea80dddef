// Host-side walk over the addressing of the matrix kernels' aligned tile loader
// (paper_1909_07588_amd/csrc/laq_tile_loader.h, the same functions the kernels compile): for every block
// tile shape the kernels instantiate, both operand orientations, contraction lengths K and widths X that
// are multiples of 4 (the fast path's precondition), every tile origin, lane and K tile,
//   * every address a lane loads 16 bytes from (uniform base + 32-bit lane offset, as the kernel forms it)
//     lies inside the operand's span of memory, and
//   * every float4 that is kept (not zeroed on the way to LDS) is the element the tile map says it is.
// The second half does the same for the softmax-regression kernel's tile loads (row-major, index-list and
// tiled sources).  Built and run by tests/test_loader_addresses.py; prints the number of addresses checked
// and of violations.
#include <cstdint>
#include <cstdio>

#include "laq_tile_loader.h"

using namespace laq;

static long long g_checked = 0, g_bad = 0;

template <int BX, int BK, bool XMAJOR>
static void walk(int X, int K, int64_t ld) {
  // an operand of K x X (K-major: S[k][x]) or X x K (X-major: S[x][k]) floats with row stride ld; the
  // loader's offsets are floats from its first element
  const int64_t span = XMAJOR ? (int64_t)(X - 1) * ld + K : (int64_t)(K - 1) * ld + X;   // floats
  using TM = TileMap<BX, BK>;
  const int n_tiles = (K + BK - 1) / BK;
  for (int x0 = 0; x0 < X; x0 += BX) {
    for (int tid = 0; tid < kLoaderThreads; ++tid) {
      FastLoaderAddr<BX, BK, XMAJOR> at;
      at.init(tid, ld, K, X, x0);
      for (int tile = 0; tile < n_tiles; ++tile) {
        const bool whole = at.is_whole(tile);
        // the uniform base the kernel hands to the buffer load lies inside the operand too
        const int64_t base = whole ? at.base(tile) : at.partial_base(tile);
        if (base < 0 || base >= span) { ++g_bad; std::printf("violation: base %lld outside span %lld\n", (long long)base, (long long)span); }
        for (int i = 0; i < TM::NV; ++i) {
          const int64_t off = whole ? at.whole(tile, i) : at.partial(tile, i);
          // the 32-bit lane offset the kernel uses reproduces it
          const uint32_t v = whole ? at.voff[i] : at.partial_voff(tile, i);
          ++g_checked;
          bool ok = off >= 0 && off + 4 <= span && (v & 15u) == 0 && base + (int64_t)(v >> 2) == off;
          if (at.keep(tile, i)) {
            int kk, xx;
            if (XMAJOR) TM::xmajor(tid, i, kk, xx); else TM::kmajor(tid, i, kk, xx);
            const int k = tile * BK + kk, x = x0 + xx;
            const int64_t want = XMAJOR ? (int64_t)x * ld + k : (int64_t)k * ld + x;
            ok = ok && TM::exists(tid, i) && k < K && x < X && off == want;
            // the whole float4 is operand data: 4 consecutive k (X-major) or x (K-major) inside the operand
            ok = ok && (XMAJOR ? k + 3 < K : x + 3 < X);
          }
          if (!ok) {
            if (g_bad < 10)
              std::printf("violation: BX=%d XMAJOR=%d X=%d K=%d ld=%lld x0=%d tid=%d tile=%d i=%d off=%lld span=%lld\n",
                          BX, (int)XMAJOR, X, K, (long long)ld, x0, tid, tile, i, (long long)off, (long long)span);
            ++g_bad;
          }
        }
      }
    }
  }
}

template <int BX>
static void shapes() {
  constexpr int BK = 16;
  // widths around one and two tiles, contractions shorter than, equal to and longer than K tiles
  const int Xs[] = {4, 8, 12, 16, 60, 64, 68, BX - 4, BX, BX + 4, 2 * BX - 4, 2 * BX, 2 * BX + 8, 200, 784, 788};
  const int Ks[] = {4, 8, 12, 16, 20, 28, 32, 36, 48, 52, 100};
  for (int X : Xs) {
    if (X < 4) continue;
    for (int K : Ks) {
      walk<BX, BK, false>(X, K, X);          // rows packed
      walk<BX, BK, false>(X, K, X + 12);     // padded rows
      walk<BX, BK, true>(X, K, K);
      walk<BX, BK, true>(X, K, K + 4);
    }
  }
}

// ------------------------------------------------------------------ softmax-regression kernel
//
// The tile loads of softmax_grad_mfma_kernel, composed here as its gaddr / gchunk / iload steps compose
// them from the shared functions: row-major source, index-list source (stochastic variant) and the tiled
// copy.  Offsets are floats from the worker's shard base (bytes for the tiled copy); every 16-byte load
// must lie inside the shard, every label and index-list read inside its array.
static long long g_smx_checked = 0, g_smx_bad = 0;

static void smx_fail(const char* what, int F, int64_t ldx, int64_t N_m, int M, int64_t r0, int wave, int lane, int n) {
  if (g_smx_bad < 10)
    std::printf("softmax violation (%s): F=%d ldx=%lld N_m=%lld M=%d r0=%lld wave=%d lane=%d n=%d\n", what, F,
                (long long)ldx, (long long)N_m, M, (long long)r0, wave, lane, n);
  ++g_smx_bad;
}

// rows: rows the blocks walk (N_m, or the minibatch size B with idx[] of that length); N_src: rows of the shard
static void walk_smx(int F, int64_t ldx, int64_t N_src, int M, int64_t rows, const int* idx, bool tiled) {
  const int NW = kSmxWavesPerBlock, RT = kSmxRowsPerTile;
  const int nchunk = (F + 15) / 16, nf4r = (F + 3) >> 2;
  int tmax, nfull;
  smx_variant(F, tiled, tmax, nfull);
  int rpb;
  const int nb = smx_blocks(256, M, rows, &rpb);
  const int64_t shard_floats = N_src * ldx;
  const int64_t tiled_bytes = ((N_src + RT - 1) / RT) * (int64_t)nchunk * 1024;
  for (int blk = 0; blk < nb; ++blk) {
    const int64_t r_begin = (int64_t)blk * rpb;
    int64_t r_end = r_begin + rpb;
    if (r_end > rows) r_end = rows;
    if (r_begin >= r_end) { smx_fail("empty block", F, ldx, N_src, M, r_begin, 0, 0, 0); continue; }
    // tiles the prologue and the loop request: r_begin, then one per step up to three tiles past the range
    for (int64_t r0 = r_begin; r0 < r_end + 3 * RT; r0 += RT) {
      const int64_t rb = smx_tile_row(r0, r_end);
      const int rows_valid = smx_rows_valid(rb, r_end);
      for (int wave = 0; wave < NW; ++wave)
        for (int lane = 0; lane < 64; ++lane) {
          const int l16 = lane & 15, lq = lane >> 4;
          const int64_t ix = rb + smx_data_row(l16, rows_valid), iy = rb + smx_label_row(wave, lq, rows_valid);
          ++g_smx_checked;
          if (ix < 0 || ix >= rows || iy < 0 || iy >= rows) smx_fail("row index", F, ldx, N_src, M, r0, wave, lane, 0);
          if (tiled) {
            const uint32_t tile_off = smx_tiled_tile_off(rb, nchunk, wave);
            for (int n = 0; n < tmax; ++n) {
              const int64_t off = (int64_t)smx_tiled_chunk_off(tile_off, n, nfull, wave, nchunk) + 16 * lane;
              ++g_smx_checked;
              if (off < 0 || off + 16 > tiled_bytes) smx_fail("tiled load", F, ldx, N_src, M, r0, wave, lane, n);
            }
            if (iy >= N_src) smx_fail("label", F, ldx, N_src, M, r0, wave, lane, 0);
            continue;
          }
          // row-major: tile base + row inside the tile; index list: the drawn row of the shard
          const int64_t base = idx ? 0 : rb * ldx;
          const uint32_t row_off = idx ? (uint32_t)idx[ix] * (uint32_t)ldx
                                       : (uint32_t)smx_data_row(l16, rows_valid) * (uint32_t)ldx;
          const int64_t ysrc = idx ? idx[iy] : iy;
          if (ysrc < 0 || ysrc >= N_src) smx_fail("label", F, ldx, N_src, M, r0, wave, lane, 0);
          const int64_t lanep = base + (int64_t)(row_off + smx_lane_col(wave, lq));
          for (int n = 0; n < tmax; ++n) {
            const int64_t off = n < nfull ? lanep + smx_chunk_step(n)
                                          : base + (int64_t)(row_off + smx_ragged_col(wave, n, lq, nf4r));
            ++g_smx_checked;
            // inside the shard, and inside its own row (columns up to ldx are the row's padding)
            const int64_t row_start = base + row_off;
            if (off < 0 || off + 4 > shard_floats || off < row_start || off + 4 > row_start + ldx)
              smx_fail("load", F, ldx, N_src, M, r0, wave, lane, n);
            // a whole chunk must hold columns below F only (it is used without a column mask)
            if (n < nfull && off - row_start + 4 > F) smx_fail("whole chunk crosses F", F, ldx, N_src, M, r0, wave, lane, n);
          }
        }
    }
  }
}

static void smx_shapes() {
  const int Fs[] = {1, 2, 3, 4, 5, 15, 16, 17, 31, 32, 33, 63, 64, 65, 255, 256, 257, 271, 272, 511, 512, 513, 527,
                    767, 768, 769, 784, 785, 800, 999, 1000, 1007, 1008};
  const int64_t Ns[] = {1, 2, 15, 16, 17, 31, 33, 100, 241, 6000};
  const int Ms[] = {1, 3, 10, 300};
  unsigned seed = 12345;
  for (int F : Fs)
    for (int pad = 0; pad < 2; ++pad) {
      const int64_t ldx = (F + 3) / 4 * 4 + 4 * pad;
      for (int64_t N_m : Ns)
        for (int M : Ms) {
          if (N_m == 6000 && (M != 10 || pad)) continue;            // the full-size workload once
          walk_smx(F, ldx, N_m, M, N_m, nullptr, false);
          if (pad == 0) walk_smx(F, ldx, N_m, M, N_m, nullptr, true);
          const int64_t B = N_m / 2 > 0 ? N_m / 2 : 1;              // a minibatch through the index list
          int* idx = new int[B];
          for (int64_t j = 0; j < B; ++j) { seed = seed * 1664525u + 1013904223u; idx[j] = (int)((seed >> 8) % (unsigned)N_m); }
          idx[0] = (int)N_m - 1;                                     // the last row of the shard is drawn
          walk_smx(F, ldx, N_m, M, B, idx, false);
          delete[] idx;
        }
    }
}

int main() {
  smx_shapes();
  std::printf("softmax kernel: checked %lld addresses, %lld violations\n", g_smx_checked, g_smx_bad);
  shapes<64>();
  shapes<128>();
  shapes<160>();
  shapes<192>();
  shapes<208>();
  shapes<224>();
  std::printf("checked %lld addresses, %lld violations\n", g_checked, g_bad);
  return g_bad == 0 && g_smx_bad == 0 ? 0 : 1;
}
