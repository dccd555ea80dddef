// Host-side walk over the addressing of the matrix kernels' aligned tile loader
// (paper_1909_07588_amd/csrc/laq_tile_loader.h, the same functions the kernels compile): for every block
// tile shape the kernels instantiate, both operand orientations, contraction lengths K and widths X that
// are multiples of 4 (the fast path's precondition), every tile origin, lane and K tile,
//   * every address a lane loads 16 bytes from lies inside the operand's span of memory, and
//   * every float4 that is kept (not zeroed on the way to LDS) is the element the tile map says it is.
// Built and run by tests/test_loader_addresses.py; prints the number of addresses checked and of violations.
#include <cstdint>
#include <cstdio>

#include "laq_tile_loader.h"

using namespace laq;

static long long g_checked = 0, g_bad = 0;

template <int BX, int BK, bool XMAJOR>
static void walk(int X, int K, int64_t ld) {
  // an operand of K x X (K-major: S[k][x]) or X x K (X-major: S[x][k]) floats with row stride ld
  float* const S = reinterpret_cast<float*>(static_cast<uintptr_t>(1) << 32);
  const int64_t span = XMAJOR ? (int64_t)(X - 1) * ld + K : (int64_t)(K - 1) * ld + X;   // floats
  using TM = TileMap<BX, BK>;
  const int n_tiles = (K + BK - 1) / BK;
  for (int x0 = 0; x0 < X; x0 += BX) {
    for (int tid = 0; tid < kLoaderThreads; ++tid) {
      FastLoaderAddr<BX, BK, XMAJOR> at;
      at.init(tid, S, ld, K, X, x0);
      for (int tile = 0; tile < n_tiles; ++tile) {
        const bool whole = at.is_whole(tile);
        for (int i = 0; i < TM::NV; ++i) {
          const float* a = whole ? at.whole(i) : at.partial(tile, i);
          const int64_t off = a - S;
          ++g_checked;
          bool ok = off >= 0 && off + 3 < span + 0 && (off + 4 <= span);
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
        if (whole) at.advance();
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

int main() {
  shapes<64>();
  shapes<128>();
  shapes<160>();
  shapes<192>();
  shapes<224>();
  std::printf("checked %lld addresses, %lld violations\n", g_checked, g_bad);
  return g_bad == 0 ? 0 : 1;
}
