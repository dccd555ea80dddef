// LAQ hot path for gfx950: context, innovation quantizer + skip rule, lazy
// aggregation + parameter update.  Algorithm 2 and eqs. 4-7 of Sun, Chen,
// Giannakis, Yang, "Communication-Efficient Distributed Learning via Lazily
// Aggregated Quantized Gradients".
//
// Data ownership per lane: 8 consecutive coordinates.  8 codes of b bits are
// exactly b bytes, so every lane writes (or reads) a whole number of bytes of
// the packed bitstream for any b and no cross-lane packing is needed; the two
// 16-byte loads per operand keep every request 16-byte aligned.
//
// This file must be compiled with -ffp-contract=off: every elementwise step
// below is one IEEE binary32 operation, in the documented order.
#include <math.h>
#include <stdarg.h>
#include <string.h>

#include <mutex>
#include <new>

#include "laq_internal.h"

namespace laq {

int set_error(laq_ctx* ctx, int status, const char* fmt, ...) {
  if (ctx) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
    va_end(ap);
  }
  return status;
}

static inline int64_t round_up(int64_t a, int64_t m) { return (a + m - 1) / m * m; }

static int32_t ceil_log2(int64_t n) {
  int32_t c = 0;
  while (((int64_t)1 << c) < n) ++c;
  return c;
}

// ------------------------------------------------------------------ device helpers

__device__ __forceinline__ uint32_t abs_bits(float d) { return __float_as_uint(d) & 0x7fffffffu; }

// Wavefront reductions; every lane gets the result.  Within each row of 16 lanes the values move
// through the data-parallel-primitive path (row_shr 1, 2, 4, 8; lanes without a source read 0), which
// costs an ordinary vector instruction per step; the four row totals (lanes 15, 31, 47, 63) are read
// into scalar registers and combined there.  A butterfly of cross-lane shuffles through LDS takes
// ~100 cycles per dependent step instead, which the small launches (one block per worker) feel.
template <int CTRL>
__device__ __forceinline__ uint32_t row_shr_u32(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}
__device__ __forceinline__ uint32_t lane_u32(uint32_t v, int lane) {
  return (uint32_t)__builtin_amdgcn_readlane((int)v, lane);
}

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
  uint32_t o;
  o = row_shr_u32<0x111>(v); v = v > o ? v : o;
  o = row_shr_u32<0x112>(v); v = v > o ? v : o;
  o = row_shr_u32<0x114>(v); v = v > o ? v : o;
  o = row_shr_u32<0x118>(v); v = v > o ? v : o;
  const uint32_t a = lane_u32(v, 15), b = lane_u32(v, 31), c = lane_u32(v, 47), d = lane_u32(v, 63);
  const uint32_t ab = a > b ? a : b, cd = c > d ? c : d;
  return ab > cd ? ab : cd;
}

template <int CTRL>
__device__ __forceinline__ unsigned long long row_shr_u64(unsigned long long v) {
  const uint32_t lo = row_shr_u32<CTRL>((uint32_t)v), hi = row_shr_u32<CTRL>((uint32_t)(v >> 32));
  return ((unsigned long long)hi << 32) | lo;
}
__device__ __forceinline__ unsigned long long lane_u64(unsigned long long v, int lane) {
  return ((unsigned long long)lane_u32((uint32_t)(v >> 32), lane) << 32) | lane_u32((uint32_t)v, lane);
}

__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long v) {
  v += row_shr_u64<0x111>(v);
  v += row_shr_u64<0x112>(v);
  v += row_shr_u64<0x114>(v);
  v += row_shr_u64<0x118>(v);
  return (lane_u64(v, 15) + lane_u64(v, 31)) + (lane_u64(v, 47) + lane_u64(v, 63));
}

// (fixed order: within a row lane 15 ends with ((x15 + x14) + (x13 + x12)) + ... , then the rows)
__device__ __forceinline__ double wave_sum_f64(double v) {
  v += __longlong_as_double((long long)row_shr_u64<0x111>((unsigned long long)__double_as_longlong(v)));
  v += __longlong_as_double((long long)row_shr_u64<0x112>((unsigned long long)__double_as_longlong(v)));
  v += __longlong_as_double((long long)row_shr_u64<0x114>((unsigned long long)__double_as_longlong(v)));
  v += __longlong_as_double((long long)row_shr_u64<0x118>((unsigned long long)__double_as_longlong(v)));
  const unsigned long long b = (unsigned long long)__double_as_longlong(v);
  const double r0 = __longlong_as_double((long long)lane_u64(b, 15)), r1 = __longlong_as_double((long long)lane_u64(b, 31));
  const double r2 = __longlong_as_double((long long)lane_u64(b, 47)), r3 = __longlong_as_double((long long)lane_u64(b, 63));
  return (r0 + r1) + (r2 + r3);
}

// Per-worker quantizer constants derived from the radius (eq. 5 denominators).
struct QuantConst {
  float R, s, step;
  int x;        // 2^(x-1) <= step < 2^x
  bool finite;  // R and 2R finite
  bool zero;    // zero (or unrepresentably small) innovation: all codes 0, delta 0
};

// B == kExact: the identity quantizer Q_m(theta^k) = grad f_m(theta^k), the limit of many
// bits in which LAQ becomes lazy aggregation of exact gradients (remark after eqs. 7a-7b).
constexpr int kExact = LAQ_B_EXACT;

template <int B>
__device__ __forceinline__ QuantConst quant_const(uint32_t rbits) {
  QuantConst c;
  c.R = __uint_as_float(rbits);
  const float two_R = 2.0f * c.R;
  c.finite = (rbits < 0x7f800000u) && (abs_bits(two_R) < 0x7f800000u);
  if constexpr (B == kExact) {
    c.s = 0.0f; c.step = 0.0f; c.x = 0;
    c.zero = !c.finite || c.R == 0.0f;
    return c;
  }
  constexpr float Lf = (float)((1u << (B & 31)) - 1u);
  // binary64 quotient of two binary32 values, rounded once more to binary32,
  // equals the correctly rounded binary32 quotient (53 >= 2*24 + 2).
  c.s = (float)((double)Lf / (double)two_R);
  c.step = (float)((double)two_R / (double)Lf);
  c.zero = !c.finite || c.R == 0.0f || !(abs_bits(c.s) < 0x7f800000u);
  c.x = 0;
  if (!c.zero) (void)frexpf(c.step, &c.x);
  return c;
}

// ------------------------------------------------------------------ sweep geometry
//
// Both streaming passes use a grid of (ceil(T/U), M) blocks: block (x, m)
// handles U consecutive tiles of 256 groups (2048 coordinates each) of worker
// m, U = 1 unless p is very large.  The hardware dispatches blocks in order
// (x fastest), so at any moment the resident blocks work on one contiguous
// window of one or two workers' rows: few concurrent DRAM streams, which is
// worth ~15 % of bandwidth on this part compared with a grid that keeps all
// workers' rows in flight.  Every block leaves its partial results in its own
// slot and a small follow-up kernel combines them: no atomics or device-scope
// fences inside the sweeps (a release fence writes back the whole L2 here and
// costs microseconds; thousands of same-address atomics serialise).

constexpr int kWavesPerBlock = kThreads / 64;
constexpr int kSoloThreads = 1024;   // block size of the one-block-per-worker launches (at most 4 tiles of 256 groups)
constexpr int kMaxSlots = 8192;   // block partials per worker

struct Sweep {
  int64_t nfull;   // whole groups of 8 coordinates per worker
  int64_t T;       // tiles of 256 groups per worker (>= 1)
  int32_t U;       // consecutive tiles per block
  int32_t Gx;      // blocks per worker
};

// ------------------------------------------------------------------ pass 1: radius

// R_m = || g_m - h_m ||_inf (Sec. 2.1).  The maximum is taken on the raw
// bits of |d| (order-free, exact, NaN > inf so a NaN is not lost).
__global__ __launch_bounds__(kThreads) void radius_kernel(const float* __restrict__ G,
                                                          const float* __restrict__ H, int64_t p,
                                                          int64_t p_stride, int32_t U, int32_t slots,
                                                          DeviceScalars sc) {
  const int64_t nfull = p / kGroup;
  {
    const int m = blockIdx.y;
    const float* g = G + (int64_t)m * p_stride;
    const float* h = H + (int64_t)m * p_stride;
    uint32_t mx = 0;
    const int64_t first = (int64_t)blockIdx.x * U * kThreads + threadIdx.x;
    for (int64_t grp = first, u = 0; u < U && grp < nfull; ++u, grp += kThreads) {
      const float4* gp = reinterpret_cast<const float4*>(g + grp * kGroup);
      const float4* hp = reinterpret_cast<const float4*>(h + grp * kGroup);
      const float4 g0 = gp[0], g1 = gp[1], h0 = hp[0], h1 = hp[1];
      uint32_t a = max(max(abs_bits(g0.x - h0.x), abs_bits(g0.y - h0.y)),
                       max(abs_bits(g0.z - h0.z), abs_bits(g0.w - h0.w)));
      uint32_t c = max(max(abs_bits(g1.x - h1.x), abs_bits(g1.y - h1.y)),
                       max(abs_bits(g1.z - h1.z), abs_bits(g1.w - h1.w)));
      mx = max(mx, max(a, c));
    }
    if (blockIdx.x == 0 && threadIdx.x == 0)
      for (int64_t i = nfull * kGroup; i < p; ++i) mx = max(mx, abs_bits(g[i] - h[i]));
    // one partial per block (the barrier comes after the block's last load)
    __shared__ uint32_t sm[kWavesPerBlock];
    mx = wave_max_u32(mx);
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = mx;
    __syncthreads();
    if (threadIdx.x == 0)
      sc.Rpart[(int64_t)m * slots + blockIdx.x] = max(max(sm[0], sm[1]), max(sm[2], sm[3]));
  }
}

// R_m from block partials src[m][0..count) (first pass, or a gradient kernel's epilogue).
__global__ __launch_bounds__(kThreads) void radius_final_kernel(const uint32_t* __restrict__ src,
                                                                int32_t stride, int32_t count,
                                                                uint32_t* __restrict__ Rfin) {
  __shared__ uint32_t sm[kThreads / 64];
  const int m = blockIdx.x;
  uint32_t mx = 0;
  // eight unconditional loads in flight per thread, from clamped indices (a repeat does not change a
  // maximum): a plain loop pays one memory latency per partial
  const uint32_t* row = src + (int64_t)m * stride;
  for (int i0 = threadIdx.x; i0 < count; i0 += 8 * kThreads) {
    uint32_t v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = row[i0 + u * kThreads < count ? i0 + u * kThreads : i0];
#pragma unroll
    for (int u = 0; u < 8; ++u) mx = max(mx, v[u]);
  }
  mx = wave_max_u32(mx);
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = mx;
  __syncthreads();
  if (threadIdx.x == 0) Rfin[m] = max(max(sm[0], sm[1]), max(sm[2], sm[3]));
}

// ------------------------------------------------------------------ pass 2: codes + skip rule

struct QuantArgs {
  const float* G;
  const float* H;
  uint32_t* codes;
  float* R_out;
  uint8_t* upload;
  DeviceScalars sc;
  int64_t p, p_stride, w_stride;
  int32_t M, D, t_bar, eps_K, slots, U;
  int32_t fused_decide;   // 1: one block per worker, which applies the skip rule itself
  // radius source: either the finished value rfin[m] (rcount == 0) or at most kDirectPartials
  // block maxima rsrc[m * rstride + i], i < rcount, combined on the fly
  const uint32_t* rsrc;
  const uint32_t* rfin;
  int32_t rstride, rcount;
  float alpha;
  uint32_t mode;
};

constexpr int kDirectPartials = 256;   // block maxima that the code pass combines itself (4 per lane)
constexpr int kMaxHistLds = 256;   // history terms staged in LDS (longer histories fall back to global reads)

// Stages xi_d * dtheta2[d] for d < min(D, kMaxHistLds) in LDS; every thread of the block calls it.
__device__ __forceinline__ void stage_history(const QuantArgs& a, double* hterm) {
  for (int d = threadIdx.x; d < a.D && d < kMaxHistLds; d += blockDim.x) hterm[d] = a.sc.xi[d] * a.sc.dtheta2[d];
}

// The skip rule (eqs. 7a-7b) for worker m in binary64 with a fixed operation order, and the
// per-call stash read by the server step; run by one thread.
__device__ __forceinline__ void apply_skip_rule(const QuantArgs& a, int m, float R, bool finite, double lhs,
                                                double E2, long long Sq, const double* hterm, double ehat2,
                                                int t_m) {
  // hterm[d] = xi_d * ||theta^{k+1-d} - theta^{k-d}||^2, fetched by D threads at once (a loop of
  // dependent global loads on one thread would cost a memory latency per term)
  double Hsum = 0.0;
  const int d_lds = a.D < kMaxHistLds ? a.D : kMaxHistLds;
  for (int d0 = 0; d0 < d_lds; d0 += 8) {          // eight reads in flight, added in ascending order
    double term[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) term[u] = hterm[d0 + u < d_lds ? d0 + u : d_lds - 1];
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (d0 + u < d_lds) Hsum = (d0 + u == 0) ? term[u] : Hsum + term[u];
  }
  for (int d = kMaxHistLds; d < a.D; ++d) Hsum = Hsum + a.sc.xi[d] * a.sc.dtheta2[d];
  const double a2 = (double)a.alpha * (double)a.alpha;
  const double m2 = (double)a.M * (double)a.M;
  const double cc = 1.0 / (a2 * m2);
  const double err = E2 + ehat2;
  const double t1 = cc * Hsum;
  const double t2 = 3.0 * err;
  const double rhs = t1 + t2;
  bool skip = (t_m < a.t_bar) && (lhs <= rhs);
  if (a.mode & LAQ_MODE_FORCE_UPLOAD) skip = false;
  if (!finite) { skip = true; atomicOr(a.sc.status, 1u); }
  a.upload[m] = skip ? 0 : 1;
  a.R_out[m] = R;
  a.sc.Sq[m] = Sq;
  a.sc.E2[m] = E2;
  a.sc.lhs[m] = lhs;
  a.sc.rhs[m] = rhs;
}

template <int B>
__device__ __forceinline__ void decide_worker(const QuantArgs& a, int m, int32_t n_slots);

// One coordinate of eqs. 5-6 plus its contributions to the two squared norms.
template <int B>
__device__ __forceinline__ uint32_t quant_one(float g, float h, const QuantConst& c, int sh,
                                              double& accN, unsigned long long& accS) {
  constexpr int L = (1 << B) - 1;
  const float d = g - h;
  const float u = d + c.R;
  float t = u * c.s;
  t = t + 0.5f;
  float qf = floorf(t);
  qf = fminf(fmaxf(qf, 0.0f), (float)L);
  const uint32_t qi = (uint32_t)qf;
  float dq = qf * c.step;
  dq = dq - c.R;
  const float hn = h + dq;
  const float e = g - hn;
  const double nd = (double)rintf(ldexpf(e, sh));   // integer-valued, |nd| < 2^21
  accN = fma(nd, nd, accN);                          // exact while accN < 2^53
  const int cc = 2 * (int)qi - L;                    // |cc| < 2^16
  // unsigned: cc^2 reaches 2^32 - 2^17 at b = 16, past the range of the signed 24-bit product
  // (whose overflow is undefined: the compiler then adds two squares in 32 bits and drops the carry)
  const uint32_t ac = (uint32_t)(cc < 0 ? -cc : cc);
  accS += (unsigned long long)(uint32_t)__umul24(ac, ac);   // (the header declares its result as int)
  return qi;
}

template <int B>
__device__ __forceinline__ void store_group(uint8_t* out, unsigned __int128 v) {
  if constexpr (B == 16) {
    uint4 w;
    w.x = (uint32_t)v; w.y = (uint32_t)(v >> 32); w.z = (uint32_t)(v >> 64); w.w = (uint32_t)(v >> 96);
    *reinterpret_cast<uint4*>(out) = w;
  } else if constexpr (B == 8) {
    uint2 w;
    w.x = (uint32_t)v; w.y = (uint32_t)(v >> 32);
    *reinterpret_cast<uint2*>(out) = w;
  } else if constexpr (B == 4) {
    *reinterpret_cast<uint32_t*>(out) = (uint32_t)v;
  } else if constexpr (B == 2) {
    *reinterpret_cast<uint16_t*>(out) = (uint16_t)v;
  } else {
#pragma unroll
    for (int k = 0; k < B; ++k) out[k] = (uint8_t)(v >> (8 * k));
  }
}

template <int B>
__device__ __forceinline__ unsigned __int128 load_group(const uint8_t* in) {
  if constexpr (B == 16) {
    const uint4 w = *reinterpret_cast<const uint4*>(in);
    return (unsigned __int128)w.x | ((unsigned __int128)w.y << 32) | ((unsigned __int128)w.z << 64) |
           ((unsigned __int128)w.w << 96);
  } else if constexpr (B == 8) {
    const uint2 w = *reinterpret_cast<const uint2*>(in);
    return (unsigned __int128)w.x | ((unsigned __int128)w.y << 32);
  } else if constexpr (B == 4) {
    return *reinterpret_cast<const uint32_t*>(in);
  } else if constexpr (B == 2) {
    return *reinterpret_cast<const uint16_t*>(in);
  } else {
    unsigned __int128 v = 0;
#pragma unroll
    for (int k = 0; k < B; ++k) v |= (unsigned __int128)in[k] << (8 * k);
    return v;
  }
}

// SOLO: one block per worker (small models; the launch is a chain of memory latencies, not
// bandwidth).  The block applies the skip rule itself and requests everything it will read before
// its first wait.  The streaming instantiation stays lean: it lives on occupancy.
template <int B, bool SOLO>
__global__ __launch_bounds__(SOLO ? kSoloThreads : kThreads) void codes_kernel(QuantArgs a) {
  constexpr int NT = SOLO ? kSoloThreads : kThreads;   // SOLO: sixteen wavefronts, one group of 8 coordinates per lane
  const int64_t nfull = a.p / kGroup;
  const int64_t first = SOLO ? (int64_t)threadIdx.x : (int64_t)blockIdx.x * a.U * kThreads + threadIdx.x;
  {
    const int m = blockIdx.y;
    const float* g = a.G + (int64_t)m * a.p_stride;
    const float* h = a.H + (int64_t)m * a.p_stride;
    uint8_t* out = reinterpret_cast<uint8_t*>(a.codes + (int64_t)m * a.w_stride);
    uint32_t rbits;
    if (a.rcount > 0) {
      // four unconditional loads from clamped indices (duplicates do not change a maximum)
      const int lane = threadIdx.x & 63;
      const uint32_t* rs = a.rsrc + (int64_t)m * a.rstride;
      const uint32_t r0 = rs[lane < a.rcount ? lane : 0], r1 = rs[lane + 64 < a.rcount ? lane + 64 : 0];
      const uint32_t r2 = rs[lane + 128 < a.rcount ? lane + 128 : 0], r3 = rs[lane + 192 < a.rcount ? lane + 192 : 0];
      rbits = max(max(r0, r1), max(r2, r3));
    } else {
      rbits = a.rfin[m];
    }
    // SOLO: everything the block will read is requested here, before the first wait: the lane's
    // group of g and h, the ragged tail, the terms of the skip rule.  The loads are
    // unconditional, from clamped addresses, and their values are not touched until used.
    constexpr bool solo = SOLO;
    const bool quick = SOLO && nfull >= 1 && nfull <= NT;
    __shared__ double hterm_s[SOLO ? kMaxHistLds : 1];
    double hx = 0.0, hd = 0.0, ehat2 = 0.0;
    int t_m = 0;
    if constexpr (SOLO) {
      const int dcl = (int)threadIdx.x < a.D ? (int)threadIdx.x : 0;
      hx = a.sc.xi[dcl]; hd = a.sc.dtheta2[dcl];
      ehat2 = a.sc.Ehat2[m];
      t_m = a.sc.t[m];
    }
    float4 qg[1][2], qh[1][2];
    float tg[kGroup - 1], th[kGroup - 1];          // the p % 8 coordinates after the last whole group
    if (quick) {
#pragma unroll
      for (int k = 0; k < kGroup - 1; ++k) {
        const int64_t i = nfull * kGroup + k < a.p ? nfull * kGroup + k : a.p - 1;
        tg[k] = g[i]; th[k] = h[i];
      }
      {
        constexpr int u = 0;
        const int64_t grp = first < nfull ? first : nfull - 1;
        const float4* gp = reinterpret_cast<const float4*>(g + grp * kGroup);
        const float4* hp = reinterpret_cast<const float4*>(h + grp * kGroup);
        qg[u][0] = gp[0]; qg[u][1] = gp[1]; qh[u][0] = hp[0]; qh[u][1] = hp[1];
      }
    }
    if (a.rcount > 0) rbits = wave_max_u32(rbits);
    const QuantConst c = quant_const<B>(rbits);
    const int sh = a.eps_K - c.x;
    double accN = 0.0;
    unsigned long long accS = 0;

    if (quick) {
      constexpr int u = 0;
      const int64_t grp = first;
      if (grp < nfull) {
        unsigned __int128 v = 0;
        if (!c.zero) {
          const float gv[8] = {qg[u][0].x, qg[u][0].y, qg[u][0].z, qg[u][0].w, qg[u][1].x, qg[u][1].y, qg[u][1].z, qg[u][1].w};
          const float hv[8] = {qh[u][0].x, qh[u][0].y, qh[u][0].z, qh[u][0].w, qh[u][1].x, qh[u][1].y, qh[u][1].z, qh[u][1].w};
#pragma unroll
          for (int j = 0; j < kGroup; ++j)
            v |= (unsigned __int128)quant_one<B>(gv[j], hv[j], c, sh, accN, accS) << (j * B);
        }
        store_group<B>(out + grp * B, v);
      }
    } else if (c.zero) {
      for (int64_t grp = first, u = 0; (SOLO || u < a.U) && grp < nfull; ++u, grp += NT)
        store_group<B>(out + grp * B, 0);
    } else {
      for (int64_t grp = first, u = 0; (SOLO || u < a.U) && grp < nfull; ++u, grp += NT) {
        const float4* gp = reinterpret_cast<const float4*>(g + grp * kGroup);
        const float4* hp = reinterpret_cast<const float4*>(h + grp * kGroup);
        const float4 g0 = gp[0], g1 = gp[1], h0 = hp[0], h1 = hp[1];
        const float gv[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
        const float hv[8] = {h0.x, h0.y, h0.z, h0.w, h1.x, h1.y, h1.z, h1.w};
        unsigned __int128 v = 0;
#pragma unroll
        for (int j = 0; j < kGroup; ++j)
          v |= (unsigned __int128)quant_one<B>(gv[j], hv[j], c, sh, accN, accS) << (j * B);
        store_group<B>(out + grp * B, v);
      }
    }
    if (solo && (int)threadIdx.x < a.D && (int)threadIdx.x < kMaxHistLds) hterm_s[threadIdx.x] = hx * hd;
    // ragged tail (p % 8 coordinates) and zero fill up to the row stride
    if (blockIdx.x == 0 && threadIdx.x == 0) {
      int64_t byte = nfull * B;
      if (a.p > nfull * kGroup) {
        unsigned __int128 v = 0;
        if (!c.zero) {
          if (quick) {
#pragma unroll
            for (int k = 0; k < kGroup - 1; ++k)
              if (nfull * kGroup + k < a.p)
                v |= (unsigned __int128)quant_one<B>(tg[k], th[k], c, sh, accN, accS) << (k * B);
          } else {
            for (int64_t i = nfull * kGroup; i < a.p; ++i)
              v |= (unsigned __int128)quant_one<B>(g[i], h[i], c, sh, accN, accS)
                   << ((int)(i - nfull * kGroup) * B);
          }
        }
        for (int k = 0; k < B; ++k) out[byte + k] = (uint8_t)(v >> (8 * k));
        byte += B;
      }
      for (; byte < a.w_stride * 4; ++byte) out[byte] = 0;
    }

    // block totals of the two exact integer sums -> slot blockIdx.x of worker m
    __shared__ unsigned long long smS[NT / 64], smN[NT / 64];
    const unsigned long long s64 = wave_sum_u64(accS);
    const unsigned long long n64 = wave_sum_u64((unsigned long long)accN);
    if ((threadIdx.x & 63) == 0) { smS[threadIdx.x >> 6] = s64; smN[threadIdx.x >> 6] = n64; }
    __syncthreads();
    if (solo) {
      if (threadIdx.x == 0) {
        constexpr int L = (1 << B) - 1;
        unsigned long long Sq = 0, N = 0;
#pragma unroll
        for (int wv = 0; wv < NT / 64; ++wv) { Sq += smS[wv]; N += smN[wv]; }
        const double E2 = c.zero ? 0.0 : ldexp((double)N, 2 * (c.x - a.eps_K));
        const double r = (double)c.R / (double)L;
        const double lhs = c.zero ? 0.0 : (r * r) * (double)(long long)Sq;
        apply_skip_rule(a, m, c.R, c.finite, lhs, E2, c.zero ? 0 : (long long)Sq, hterm_s, ehat2, t_m);
      }
      return;
    }
    // Several blocks per worker: each leaves its partials in its own slot and decide_kernel
    // combines them.  (Letting the last block to finish do that behind a device-scope fence and a
    // counter was measured: 29 vs 15 us at M = 10, p = 120 000 and 172 vs 30 us at M = 64.)
    if (threadIdx.x == 0) {
      const int64_t slot = (int64_t)m * a.slots + blockIdx.x;
      a.sc.Spart[slot] = (smS[0] + smS[1]) + (smS[2] + smS[3]);
      a.sc.Npart[slot] = (smN[0] + smN[1]) + (smN[2] + smN[3]);
    }
  }
}

// Totals of the block partials (integers: order-free) and the skip rule
// (eqs. 7a-7b) in binary64 with a fixed operation order; run by one block for worker m.
template <int B>
__device__ __forceinline__ void decide_worker(const QuantArgs& a, int m, int32_t n_slots) {
  constexpr int L = (1 << B) - 1;
  __shared__ unsigned long long smS[kThreads / 64], smN[kThreads / 64];
  __shared__ uint32_t smR[kThreads / 64];
  __shared__ double hterm[kMaxHistLds];
  stage_history(a, hterm);
  unsigned long long s64 = 0, n64 = 0;
  uint32_t rb = 0;
  // Four slots of each sum in flight per thread (unconditional loads from clamped indices; the sums
  // are integers, so the order is free): a plain loop pays a memory latency per slot.
  const unsigned long long* Sp = a.sc.Spart + (int64_t)m * a.slots;
  const unsigned long long* Np = a.sc.Npart + (int64_t)m * a.slots;
  for (int i0 = threadIdx.x; i0 < n_slots; i0 += 4 * kThreads) {
    unsigned long long sv[4], nv[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = i0 + u * kThreads < n_slots ? i0 + u * kThreads : i0;
      sv[u] = Sp[i]; nv[u] = Np[i];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (i0 + u * kThreads < n_slots) { s64 += sv[u]; n64 += nv[u]; }
  }
  if (a.rcount > 0) {
    if ((int)threadIdx.x < a.rcount) rb = a.rsrc[(int64_t)m * a.rstride + threadIdx.x];
  } else if (threadIdx.x == 0) {
    rb = a.rfin[m];
  }
  s64 = wave_sum_u64(s64);
  n64 = wave_sum_u64(n64);
  rb = wave_max_u32(rb);
  if ((threadIdx.x & 63) == 0) { smS[threadIdx.x >> 6] = s64; smN[threadIdx.x >> 6] = n64; smR[threadIdx.x >> 6] = rb; }
  __syncthreads();
  if (threadIdx.x != 0) return;
  const unsigned long long Sq = smS[0] + smS[1] + smS[2] + smS[3];
  const unsigned long long N = smN[0] + smN[1] + smN[2] + smN[3];
  const QuantConst c = quant_const<B>(max(max(smR[0], smR[1]), max(smR[2], smR[3])));
  const double E2 = c.zero ? 0.0 : ldexp((double)N, 2 * (c.x - a.eps_K));
  const double r = (double)c.R / (double)L;
  const double lhs = c.zero ? 0.0 : (r * r) * (double)(long long)Sq;
  apply_skip_rule(a, m, c.R, c.finite, lhs, E2, c.zero ? 0 : (long long)Sq, hterm, a.sc.Ehat2[m], a.sc.t[m]);
}

template <int B>
__global__ __launch_bounds__(kThreads) void decide_kernel(QuantArgs a, int32_t n_slots) {
  decide_worker<B>(a, blockIdx.x, n_slots);
}

// ------------------------------------------------------------------ identity quantizer (b = LAQ_B_EXACT)
//
// One pass: the message of worker m is grad f_m itself (32 p bits), so nothing
// depends on the radius; the pass copies g into the message buffer and leaves, per
// block, max |g - h| and the binary64 sum of (g - h)^2 (each square is exact in
// binary64; lanes add sequentially, then a wavefront tree, then the four waves).
__global__ __launch_bounds__(kThreads) void exact_message_kernel(QuantArgs a) {
  const int64_t nfull = a.p / kGroup;
  const int64_t first = (int64_t)blockIdx.x * a.U * kThreads + threadIdx.x;
  const int m = blockIdx.y;
  const float* g = a.G + (int64_t)m * a.p_stride;
  const float* h = a.H + (int64_t)m * a.p_stride;
  float* out = reinterpret_cast<float*>(a.codes + (int64_t)m * a.w_stride);
  uint32_t mx = 0;
  double acc = 0.0;
  for (int64_t grp = first, u = 0; u < a.U && grp < nfull; ++u, grp += kThreads) {
    const float4* gp = reinterpret_cast<const float4*>(g + grp * kGroup);
    const float4* hp = reinterpret_cast<const float4*>(h + grp * kGroup);
    const float4 g0 = gp[0], g1 = gp[1], h0 = hp[0], h1 = hp[1];
    const float gv[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
    const float hv[8] = {h0.x, h0.y, h0.z, h0.w, h1.x, h1.y, h1.z, h1.w};
#pragma unroll
    for (int j = 0; j < kGroup; ++j) {
      const float d = gv[j] - hv[j];
      mx = max(mx, abs_bits(d));
      acc = fma((double)d, (double)d, acc);
    }
    float4* op = reinterpret_cast<float4*>(out + grp * kGroup);
    op[0] = g0;
    op[1] = g1;
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    int64_t i = nfull * kGroup;
    for (; i < a.p; ++i) {
      const float d = g[i] - h[i];
      mx = max(mx, abs_bits(d));
      acc = fma((double)d, (double)d, acc);
      out[i] = g[i];
    }
    for (; i < a.w_stride; ++i) out[i] = 0.0f;
  }
  __shared__ uint32_t smR[kWavesPerBlock];
  __shared__ double smD[kWavesPerBlock];
  mx = wave_max_u32(mx);
  acc = wave_sum_f64(acc);
  if ((threadIdx.x & 63) == 0) { smR[threadIdx.x >> 6] = mx; smD[threadIdx.x >> 6] = acc; }
  __syncthreads();
  if (threadIdx.x == 0) {
    const int64_t slot = (int64_t)m * a.slots + blockIdx.x;
    a.sc.Rpart[slot] = max(max(smR[0], smR[1]), max(smR[2], smR[3]));
    a.sc.Npart[slot] = (unsigned long long)__double_as_longlong((smD[0] + smD[1]) + (smD[2] + smD[3]));
  }
}

// ||g_m - h_m||^2 from the block partials (strided per thread, then a tree: a fixed order), the
// radius, and the skip rule with eps = 0; one block per worker.
__global__ __launch_bounds__(kThreads) void exact_decide_kernel(QuantArgs a, int32_t n_slots) {
  __shared__ double red[kThreads];
  __shared__ uint32_t smR[kWavesPerBlock];
  __shared__ double hterm[kMaxHistLds];
  stage_history(a, hterm);
  const int m = blockIdx.x;
  double tot = 0.0;
  uint32_t rb = 0;
  for (int i = threadIdx.x; i < n_slots; i += kThreads) {
    tot += __longlong_as_double((long long)a.sc.Npart[(int64_t)m * a.slots + i]);
    rb = max(rb, a.sc.Rpart[(int64_t)m * a.slots + i]);
  }
  red[threadIdx.x] = tot;
  rb = wave_max_u32(rb);
  if ((threadIdx.x & 63) == 0) smR[threadIdx.x >> 6] = rb;
  __syncthreads();
  for (int off = kThreads / 2; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x != 0) return;
  const QuantConst c = quant_const<kExact>(max(max(smR[0], smR[1]), max(smR[2], smR[3])));
  apply_skip_rule(a, m, c.R, c.finite, c.finite ? red[0] : 0.0, 0.0, 0, hterm, a.sc.Ehat2[m], a.sc.t[m]);
}

// ------------------------------------------------------------------ server step

struct ServerArgs {
  const uint32_t* codes;
  const float* R_in;
  const uint8_t* upload;
  float* H;
  float* nabla;
  float* theta;
  DeviceScalars sc;
  int64_t p, p_stride, w_stride;
  int32_t M, D, b, J;
  int32_t fused_finish;   // 1: the last block to finish does the bookkeeping (small grids)
  float alpha;
};

// First chunk (index threadIdx.x) of every array the bookkeeping reads, fetched in one go so that
// the block pays one memory latency for them, not one per array.
struct FinishFetch {
  double e2, part, older;
  unsigned long long n_uploads;
  int32_t t;
  uint8_t up;
};

// own_total: the sum of ||nabla||^2 when the calling block is the whole grid (then no partial is read)
__device__ __forceinline__ FinishFetch finish_fetch(const ServerArgs& a, int n_blocks, bool own_total) {
  // Every load is unconditional, from an index clamped into its array, and nothing here looks at a
  // loaded value: a load under a branch, or one whose value is used at once, makes the thread wait
  // for it on the spot, and the block would pay one memory latency per array again.
  FinishFetch f;
  const int m = threadIdx.x;
  const int mc = m < a.M ? m : a.M - 1;
  f.up = a.upload[mc];
  f.e2 = a.sc.E2[mc];
  f.t = a.sc.t[mc];
  f.n_uploads = a.sc.uploads[mc];
  f.part = 0.0;
  if (!own_total)
    f.part = __hip_atomic_load(&a.sc.srv_part[m < n_blocks ? m : n_blocks - 1], __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
  const int d = a.D - 1 - m;
  f.older = a.sc.dtheta2[d >= 1 ? d - 1 : 0];
  return f;
}

template <int B, int NT>
__device__ __forceinline__ void server_finish(const ServerArgs& a, int n_blocks, const FinishFetch& f,
                                              const double* own_total);

constexpr int kServerJ = 4;   // groups of 8 coordinates owned by one lane, at most
constexpr int kServerList = 4096;   // workers per round of the server step (12 bytes of LDS each)

// eq. 4: nabla^k = nabla^{k-1} + sum_{m in M^k} deltaQ_m, theta^{k+1} = theta^k - alpha nabla^k,
// with Q_m(theta_hat_m) += deltaQ_m for the uploading workers (Alg. 2, upload branch).
// Worker-major: a lane owns up to 4 groups of 8 coordinates for the whole
// kernel and keeps their running sums in registers, so the grid sweeps one
// uploading worker's row at a time (one read stream, one write stream) in
// ascending m -- the order in which the sums are defined.  A block's J NT
// groups are one contiguous stretch of the row (its J slices side by side:
// 5.10 TB/s in a full round of 64 workers x 2^24 coordinates, against 4.96 with
// the slices a whole grid apart and 4.99 with blocks of 1024 threads).
// SOLO: the grid is this one block. It then fetches nabla, theta and what the bookkeeping reads
// at the start, so that a call on a small model pays for three dependent memory round trips
// (upload flags, message rows, stores) instead of seven.
template <int B, bool SOLO>
__global__ __launch_bounds__(SOLO ? kSoloThreads : kThreads) void server_kernel(ServerArgs a) {
  constexpr int NT = SOLO ? kSoloThreads : kThreads;   // SOLO: sixteen wavefronts, one group of 8 coordinates per lane
  constexpr int JN = SOLO ? 1 : kServerJ;
  constexpr uint32_t L = B >= 32 ? 0xffffffffu : (1u << (B & 31)) - 1u;
  extern __shared__ unsigned char smem_raw[];
  const int lcap = a.M < kServerList ? a.M : kServerList;
  int32_t* list = reinterpret_cast<int32_t*>(smem_raw);           // [lcap] uploading workers of a round, ascending
  float* Rm = reinterpret_cast<float*>(list + lcap);              // [lcap]
  float* stepm = Rm + lcap;                                       // [lcap]
  __shared__ int n_up_s;

  const int64_t nfull = a.p / kGroup;
  const int64_t span = NT;                                             // slice j of the block's stretch
  const int64_t grp0 = (int64_t)blockIdx.x * a.J * NT + threadIdx.x;
  float4 pn[JN][2], pt[JN][2];
  float tn[kGroup - 1], tt[kGroup - 1];            // the p % 8 coordinates after the last whole group
  FinishFetch ff;
  if constexpr (SOLO) {
    ff = finish_fetch(a, 1, true);
#pragma unroll
    for (int k = 0; k < kGroup - 1; ++k) {
      const int64_t i = nfull * kGroup + k < a.p ? nfull * kGroup + k : a.p - 1;
      tn[k] = a.nabla[i]; tt[k] = a.theta[i];
    }
#pragma unroll
    for (int j = 0; j < JN; ++j) {
      const int64_t grp = grp0 + j * span;
      if (j < a.J && grp < nfull) {
        const float4* np4 = reinterpret_cast<const float4*>(a.nabla + grp * kGroup);
        const float4* tp4 = reinterpret_cast<const float4*>(a.theta + grp * kGroup);
        pn[j][0] = np4[0]; pn[j][1] = np4[1]; pt[j][0] = tp4[0]; pt[j][1] = tp4[1];
      }
    }
  }

  // Uploading workers are taken in ascending rounds of at most kServerList workers, so the LDS need
  // does not grow with M; inside a round: the ascending list of workers whose message carries a
  // non-zero innovation (order-preserving compaction: wavefront ballots + prefix counts).
  __shared__ int wave_cnt[NT / 64];
  float acc[JN][kGroup];
#pragma unroll
  for (int j = 0; j < JN; ++j)
#pragma unroll
    for (int i = 0; i < kGroup; ++i) acc[j][i] = 0.0f;
  float acc_tail[kGroup - 1];                      // wavefront 0 of block 0: the p % 8 last coordinates
#pragma unroll
  for (int k = 0; k < kGroup - 1; ++k) acc_tail[k] = 0.0f;

  for (int m0 = 0; m0 < a.M; m0 += kServerList) {
    const int mcnt = a.M - m0 < kServerList ? a.M - m0 : kServerList;
    if (threadIdx.x == 0) n_up_s = 0;
    for (int base = 0; base < mcnt; base += NT) {
      const int ml = base + threadIdx.x;             // index inside the round
      bool on = false;
      if (ml < mcnt) {
        const float R = a.R_in[m0 + ml];
        const QuantConst c = quant_const<B>(__float_as_uint(R));
        Rm[ml] = R;
        on = a.upload[m0 + ml] && (B == kExact || !c.zero);   // the exact message is stored even if it repeats h
        stepm[ml] = on ? c.step : -1.0f;
      }
      const unsigned long long bal = __ballot(on);
      const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
      if (lane == 0) wave_cnt[wave] = __popcll(bal);
      __syncthreads();
      int before = n_up_s;
      for (int wv = 0; wv < wave; ++wv) before += wave_cnt[wv];
      if (on) list[before + __popcll(bal & ((1ull << lane) - 1ull))] = ml;
      __syncthreads();
      if (threadIdx.x == 0) {
        int tot = 0;
#pragma unroll
        for (int wv = 0; wv < NT / 64; ++wv) tot += wave_cnt[wv];
        n_up_s += tot;
      }
      __syncthreads();
    }
    const int n_up = n_up_s;

    for (int k = 0; k < n_up; ++k) {
      const int ml = list[k];
      const int m = m0 + ml;
      const float R = Rm[ml], step = stepm[ml];
      const uint8_t* crow = reinterpret_cast<const uint8_t*>(a.codes + (int64_t)m * a.w_stride);
      float* hrow = a.H + (int64_t)m * a.p_stride;
#pragma unroll
      for (int j = 0; j < JN; ++j) {
        const int64_t grp = grp0 + j * span;
        if (j < a.J && grp < nfull) {
          float4* hp = reinterpret_cast<float4*>(hrow + grp * kGroup);
          const float4 h0 = hp[0], h1 = hp[1];
          float hv[8] = {h0.x, h0.y, h0.z, h0.w, h1.x, h1.y, h1.z, h1.w};
          if constexpr (B == kExact) {
            const float4* cp = reinterpret_cast<const float4*>(crow + grp * (int64_t)(kGroup * 4));
            const float4 g0 = cp[0], g1 = cp[1];
            const float gv[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
#pragma unroll
            for (int i = 0; i < kGroup; ++i) {
              const float dq = gv[i] - hv[i];
              hv[i] = gv[i];
              acc[j][i] = acc[j][i] + dq;
            }
          } else {
            const unsigned __int128 v = load_group<B>(crow + grp * B);
#pragma unroll
            for (int i = 0; i < kGroup; ++i) {
              const uint32_t q = (uint32_t)(v >> (i * B)) & L;
              float dq = (float)q * step;
              dq = dq - R;
              hv[i] = hv[i] + dq;
              acc[j][i] = acc[j][i] + dq;
            }
          }
          hp[0] = make_float4(hv[0], hv[1], hv[2], hv[3]);
          hp[1] = make_float4(hv[4], hv[5], hv[6], hv[7]);
        }
      }
    }
    // The p % 8 coordinates after the last whole group: wavefront 0 of block 0.  Lane l takes the
    // l-th uploader of a group of 64 (all their loads are in flight together; one thread walking the
    // uploaders would pay two memory latencies for each), then the contributions are added in
    // ascending worker order.
    if (blockIdx.x == 0 && threadIdx.x < 64) {
      const int lane = threadIdx.x;
#pragma unroll
      for (int kt = 0; kt < kGroup - 1; ++kt) {
        const int64_t i = nfull * kGroup + kt;
        if (i >= a.p) break;
        float acc1 = acc_tail[kt];
        for (int k0 = 0; k0 < n_up; k0 += 64) {
          const int k = k0 + lane;
          float dq = 0.0f;
          if (k < n_up) {
            const int ml = list[k];
            const int m = m0 + ml;
            const uint8_t* row = reinterpret_cast<const uint8_t*>(a.codes + (int64_t)m * a.w_stride);
            float* hp = a.H + (int64_t)m * a.p_stride + i;
            if constexpr (B == kExact) {
              const float gval = reinterpret_cast<const float*>(row)[i];
              dq = gval - *hp;
              *hp = gval;
            } else {
              const int64_t bit = i * B;
              uint32_t q = 0;
              for (int t = 0; t < B; ++t) q |= (uint32_t)((row[(bit + t) >> 3] >> ((bit + t) & 7)) & 1u) << t;
              dq = (float)q * stepm[ml];
              dq = dq - Rm[ml];
              *hp = *hp + dq;
            }
          }
          const int cnt = n_up - k0 < 64 ? n_up - k0 : 64;
          for (int l = 0; l < cnt; ++l)
            acc1 = acc1 + __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, dq), l));
        }
        acc_tail[kt] = acc1;
      }
    }
    __syncthreads();                                 // the next round rewrites the list
  }

  double n2 = 0.0;
#pragma unroll
  for (int j = 0; j < JN; ++j) {
    const int64_t grp = grp0 + j * span;
    if (j < a.J && grp < nfull) {
      float4* np4 = reinterpret_cast<float4*>(a.nabla + grp * kGroup);
      float4* tp4 = reinterpret_cast<float4*>(a.theta + grp * kGroup);
      float4 n0, n1, t0, t1;
      if constexpr (SOLO) {
        n0 = pn[j][0]; n1 = pn[j][1]; t0 = pt[j][0]; t1 = pt[j][1];
      } else {
        n0 = np4[0]; n1 = np4[1]; t0 = tp4[0]; t1 = tp4[1];
      }
      float nv[8] = {n0.x, n0.y, n0.z, n0.w, n1.x, n1.y, n1.z, n1.w};
      float tv[8] = {t0.x, t0.y, t0.z, t0.w, t1.x, t1.y, t1.z, t1.w};
#pragma unroll
      for (int i = 0; i < kGroup; ++i) {
        const float nb = nv[i] + acc[j][i];
        nv[i] = nb;
        const float st = a.alpha * nb;
        tv[i] = tv[i] - st;
        n2 = fma((double)nb, (double)nb, n2);
      }
      np4[0] = make_float4(nv[0], nv[1], nv[2], nv[3]);
      np4[1] = make_float4(nv[4], nv[5], nv[6], nv[7]);
      tp4[0] = make_float4(tv[0], tv[1], tv[2], tv[3]);
      tp4[1] = make_float4(tv[4], tv[5], tv[6], tv[7]);
    }
  }
  // the p % 8 last coordinates: their sums over the uploaders were formed above (wavefront 0 of block 0)
  if (blockIdx.x == 0 && threadIdx.x == 0) {
#pragma unroll
    for (int kt = 0; kt < kGroup - 1; ++kt) {
      const int64_t i = nfull * kGroup + kt;
      if (i >= a.p) break;
      float nb_old, th_old;
      if constexpr (SOLO) {                          // fetched at the start of the kernel
        nb_old = tn[kt]; th_old = tt[kt];
      } else {
        nb_old = a.nabla[i]; th_old = a.theta[i];
      }
      const float nb = nb_old + acc_tail[kt];
      a.nabla[i] = nb;
      const float st = a.alpha * nb;
      a.theta[i] = th_old - st;
      n2 = fma((double)nb, (double)nb, n2);
    }
  }

  n2 = wave_sum_f64(n2);
  __shared__ double smd[NT / 64];
  __shared__ bool last_s;
  if ((threadIdx.x & 63) == 0) smd[threadIdx.x >> 6] = n2;
  __syncthreads();
  if constexpr (SOLO) {
    __shared__ double total_s;
    if (threadIdx.x == 0) {
      double tot = 0.0;
#pragma unroll
      for (int wv = 0; wv < NT / 64; ++wv) tot += smd[wv];   // fixed order
      total_s = tot;
    }
    __syncthreads();
    server_finish<B, NT>(a, 1, ff, &total_s);
  } else {
    if (threadIdx.x == 0) {
      double tot = 0.0;
#pragma unroll
      for (int wv = 0; wv < NT / 64; wv += 4) tot += (smd[wv] + smd[wv + 1]) + (smd[wv + 2] + smd[wv + 3]);   // fixed order
      a.sc.srv_part[blockIdx.x] = tot;
      if (a.fused_finish) {
        __threadfence();
        last_s = (atomicAdd(a.sc.srv_ticket, 1u) == gridDim.x - 1);
      }
    }
    if (!a.fused_finish) return;      // large grids: a follow-up kernel finishes (no fences here)
    __syncthreads();
    if (!last_s) return;
    __threadfence();
    if (threadIdx.x == 0) *a.sc.srv_ticket = 0;
    server_finish<B, NT>(a, (int)gridDim.x, finish_fetch(a, (int)gridDim.x, false), nullptr);
  }
}

// Bookkeeping of Algorithm 2 (clocks, error norms, counters) and the new entry
// alpha^2 ||nabla||^2 of the parameter-difference history; run by one block.
template <int B, int NT>
__device__ __forceinline__ void server_finish(const ServerArgs& a, int n_blocks, const FinishFetch& f,
                                              const double* own_total) {
  __shared__ double red[NT];
  unsigned long long my_bits = 0;
  const unsigned long long msg_bits = (B == kExact ? 0ull : 32ull) + (unsigned long long)B * (unsigned long long)a.p;
  if ((int)threadIdx.x < a.M) {                       // first chunk: already fetched
    const int m = threadIdx.x;
    if (f.up) {
      a.sc.Ehat2[m] = f.e2;
      a.sc.t[m] = 0;
      a.sc.uploads[m] = f.n_uploads + 1;
      my_bits += msg_bits;
    } else {
      a.sc.t[m] = f.t + 1;
    }
  }
  for (int m = threadIdx.x + NT; m < a.M; m += NT) {
    if (a.upload[m]) {
      a.sc.Ehat2[m] = a.sc.E2[m];
      a.sc.t[m] = 0;
      a.sc.uploads[m] += 1;
      my_bits += msg_bits;
    } else {
      a.sc.t[m] += 1;
    }
  }
  if (my_bits) atomicAdd(a.sc.bits, my_bits);
  // ||nabla||^2: block partials summed in a fixed order (strided, then a tree); the one-block launch
  // brings its own total
  double total;
  if (own_total) {
    total = *own_total;
  } else {
    double tot = (int)threadIdx.x < n_blocks ? f.part : 0.0;
    for (int i = threadIdx.x + NT; i < n_blocks; i += NT)
      tot += __hip_atomic_load(&a.sc.srv_part[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    red[threadIdx.x] = tot;
    __syncthreads();
    for (int off = NT / 2; off > 0; off >>= 1) {
      if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
      __syncthreads();
    }
    total = red[0];
  }
  // history shift: all entries are read before any is written (one memory latency, not D)
  const double newest = ((double)a.alpha * (double)a.alpha) * total;
  bool first = true;
  for (int base = a.D - 1; base >= 0; base -= NT) {        // highest chunk first
    const int d = base - (int)threadIdx.x;                       // this thread's destination
    double v = 0.0;
    if (first) v = f.older;                                      // fetched before anything was written (used if d >= 1)
    else if (d >= 1) v = a.sc.dtheta2[d - 1];
    first = false;
    __syncthreads();
    if (d >= 1) a.sc.dtheta2[d] = v;
    else if (d == 0) a.sc.dtheta2[0] = newest;
    __syncthreads();
  }
}

template <int B>
__global__ __launch_bounds__(kThreads) void server_finish_kernel(ServerArgs a, int n_blocks) {
  server_finish<B, kThreads>(a, n_blocks, finish_fetch(a, n_blocks, false), nullptr);
}

__global__ void fill_i32_kernel(int32_t* p, int32_t v, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// ------------------------------------------------------------------ host side

struct Layout {
  size_t H, nabla, scalars, total;
  size_t Rpart, Spart, Npart, Rfin, Rhand, Sq, E2, lhs, rhs, Ehat2, t, uploads, bits, status, srv_ticket,
      dtheta2, xi, srv_part, scalars_end;
};

// Server step: J groups per lane (at most kServerJ), enough blocks to cover p.
static int64_t server_blocks(int64_t p, int32_t* J_out) {
  const int64_t nfull = p / kGroup;
  int64_t T = (nfull + kThreads - 1) / kThreads;
  if (T < 1) T = 1;
  int64_t J = (T + 2047) / 2048;
  if (T <= kServerJ) J = T;          // small problems: one block, no hand-over between blocks
  if (J > kServerJ) J = kServerJ;
  if (J < 1) J = 1;
  if (J_out) *J_out = (int32_t)J;
  return (T + J - 1) / J;
}

// Upper bound of block-partial slots per worker in the two streaming passes.
static int32_t partial_slots(int32_t M) {
  if (M <= 64) return kMaxSlots;
  const int32_t s = 524288 / M;
  return s < 32 ? 32 : s;
}

// Grid of the two streaming passes: Gx blocks per worker (at most max_gx), U tiles per block.
static Sweep make_sweep(int64_t p, int64_t max_gx) {
  Sweep sw;
  sw.nfull = p / kGroup;
  sw.T = (sw.nfull + kThreads - 1) / kThreads;
  if (sw.T < 1) sw.T = 1;
  sw.U = (int32_t)((sw.T + max_gx - 1) / max_gx);
  if (sw.T <= 4) sw.U = (int32_t)sw.T;   // small problems: one block per worker finishes its own skip test
  sw.Gx = (int32_t)((sw.T + sw.U - 1) / sw.U);
  return sw;
}

// Slots actually used (and allocated) per worker.
static int32_t used_slots(int64_t p, int32_t M) { return make_sweep(p, partial_slots(M)).Gx; }

static Layout make_layout(int32_t M, int64_t p, int32_t D) {
  Layout l{};
  const int64_t ps = laq_p_stride(p);
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = (size_t)round_up((int64_t)(off + bytes), 256); return o; };
  l.H = take((size_t)M * ps * sizeof(float));
  l.nabla = take((size_t)ps * sizeof(float));
  l.scalars = off;
  const size_t slots = (size_t)used_slots(p, M);
  l.Rpart = take((size_t)M * slots * 4);
  l.Spart = take((size_t)M * slots * 8);
  l.Npart = take((size_t)M * slots * 8);
  l.Rfin = take((size_t)M * 4);
  l.Rhand = take((size_t)M * 4);
  l.Sq = take((size_t)M * 8);
  l.E2 = take((size_t)M * 8);
  l.lhs = take((size_t)M * 8);
  l.rhs = take((size_t)M * 8);
  l.Ehat2 = take((size_t)M * 8);
  l.t = take((size_t)M * 4);
  l.uploads = take((size_t)M * 8);
  l.bits = take(8);
  l.status = take(4);
  l.srv_ticket = take(4);
  l.dtheta2 = take((size_t)D * 8);
  l.xi = take((size_t)D * 8);
  l.srv_part = take((size_t)server_blocks(p, nullptr) * 8);
  l.scalars_end = off;
  l.total = off;
  return l;
}

static bool valid_sizes(int32_t M, int64_t p, int32_t b, int32_t D) {
  if (!(M >= 1 && M <= 65535 && p >= 1 && p < ((int64_t)1 << 31) && ((b >= 1 && b <= LAQ_MAX_BITS) || b == LAQ_B_EXACT) &&
        D >= 1 && D <= 4096))
    return false;
  // every lane handles at most 512 groups of 8 coordinates per pass
  return p / kGroup <= (int64_t)partial_slots(M) * kThreads * 512;
}

template <int B>
static void launch_codes(dim3 grid, hipStream_t s, const QuantArgs& a) {
  if (grid.x == 1 && a.fused_decide) {
    hipLaunchKernelGGL((codes_kernel<B, true>), grid, dim3(kSoloThreads), 0, s, a);
    return;
  }
  hipLaunchKernelGGL((codes_kernel<B, false>), grid, dim3(kThreads), 0, s, a);
  if (!a.fused_decide)
    hipLaunchKernelGGL(decide_kernel<B>, dim3((unsigned)a.M), dim3(kThreads), 0, s, a, (int32_t)grid.x);
}
template <int B>
static void launch_server(dim3 grid, size_t smem, hipStream_t s, const ServerArgs& a) {
  if (grid.x == 1) {
    ServerArgs a1 = a;
    a1.J = 1;                                   // 1024 lanes cover the at most 1024 groups of 8 coordinates
    hipLaunchKernelGGL((server_kernel<B, true>), grid, dim3(kSoloThreads), smem, s, a1);
    return;
  }
  hipLaunchKernelGGL((server_kernel<B, false>), grid, dim3(kThreads), smem, s, a);
  if (!a.fused_finish)
    hipLaunchKernelGGL(server_finish_kernel<B>, dim3(1), dim3(kThreads), 0, s, a, (int)grid.x);
}

#define LAQ_DISPATCH_B(b, CALL)                                                                   \
  switch (b) {                                                                                    \
    case 1: CALL(1); break;   case 2: CALL(2); break;   case 3: CALL(3); break;                    \
    case 4: CALL(4); break;   case 5: CALL(5); break;   case 6: CALL(6); break;                    \
    case 7: CALL(7); break;   case 8: CALL(8); break;   case 9: CALL(9); break;                    \
    case 10: CALL(10); break; case 11: CALL(11); break; case 12: CALL(12); break;                  \
    case 13: CALL(13); break; case 14: CALL(14); break; case 15: CALL(15); break;                  \
    case 16: CALL(16); break;                                                                     \
    default: break;                                                                               \
  }

// Minibatch rows of every worker, copied out of the resident shards:
// Xb[m][j][:] = X[m][idx[m][j]][:], yb[m][j] = y[m][idx[m][j]].  One float4 per
// thread.  An index outside [0, N_m) is clamped (no access leaves the shard)
// and reported through the status word.
__global__ __launch_bounds__(kThreads) void gather_rows_kernel(
    const float* __restrict__ X, const int32_t* __restrict__ y, const int32_t* __restrict__ idx,
    int64_t N_m, int64_t ldx, int64_t B, float* __restrict__ Xb, int32_t* __restrict__ yb,
    uint32_t* __restrict__ status) {
  const int m = blockIdx.y;
  const int64_t nf4 = ldx >> 2;
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= B * nf4) return;
  const int64_t j = i / nf4, c4 = i - j * nf4;
  int64_t n = idx[(int64_t)m * B + j];
  if (n < 0 || n >= N_m) {
    if (c4 == 0) atomicOr(status, 2u);
    n = n < 0 ? 0 : N_m - 1;
  }
  const float4 v = *reinterpret_cast<const float4*>(X + ((int64_t)m * N_m + n) * ldx + 4 * c4);
  *reinterpret_cast<float4*>(Xb + ((int64_t)m * B + j) * ldx + 4 * c4) = v;
  if (c4 == 0) yb[(int64_t)m * B + j] = y[(int64_t)m * N_m + n];
}

// layout of the minibatch workspace: gathered rows, gathered labels, model scratch for B samples
struct MinibatchLayout {
  size_t Xb, yb, model, total;
};
static MinibatchLayout minibatch_layout(const laq_ctx* ctx, int64_t B) {
  MinibatchLayout l{};
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t at = off; off += (bytes + 255) & ~(size_t)255; return at; };
  l.Xb = take((size_t)ctx->M * (size_t)B * (size_t)ctx->ldx * sizeof(float));
  l.yb = take((size_t)ctx->M * (size_t)B * sizeof(int32_t));
  l.model = take(model_workspace_bytes(ctx, B));
  l.total = off;
  return l;
}

// ------------------------------------------------------------------ static scratch (laq_quantize_skip_noalloc)
//
// Block partials of the two streaming passes for callers that bring no scratch memory: a
// file-scope device array, one copy per GPU, held until the process ends.  In host code the
// array's name is only a handle; its device address comes from hipGetSymbolAddress, once per
// device (resolve_static_scratch), and host code uses that address everywhere.
constexpr int kStaticSlots = 65536;   // block partials in all (M * blocks per worker)
constexpr int kStaticMaxM = 4096;     // workers
struct StaticScratch {
  unsigned long long Spart[kStaticSlots];
  unsigned long long Npart[kStaticSlots];
  uint32_t Rpart[kStaticSlots];
  uint32_t Rfin[kStaticMaxM];
};
static __device__ __align__(256) unsigned char scratch[sizeof(StaticScratch)];

constexpr int kMaxDevices = 64;
static unsigned char* g_scratch_ptr[kMaxDevices] = {nullptr};
static std::mutex g_scratch_mutex;

// Device address of this GPU's copy of the array; `device` must be the current device.
static hipError_t resolve_static_scratch(int device, unsigned char** out) {
  *out = nullptr;
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[device] = static_cast<unsigned char*>(ptr);
  }
  *out = g_scratch_ptr[device];
  return hipSuccess;
}

}  // namespace laq

using namespace laq;

extern "C" {

int64_t laq_p_stride(int64_t p) { return round_up(p, 4); }

int64_t laq_w_stride(int64_t p, int32_t b) {
  const int64_t groups = (p + kGroup - 1) / kGroup;
  const int64_t bytes = groups * b;
  return round_up(bytes, 16) / 4;
}

size_t laq_workspace_bytes(int32_t M, int64_t p, int32_t b, int32_t D) {
  if (!valid_sizes(M, p, b, D)) return 0;
  return make_layout(M, p, D).total;
}

int laq_reset(laq_ctx* ctx) {
  if (!ctx) return LAQ_EINVAL;
  ctx->radius_for = nullptr;
  const Layout l = make_layout(ctx->M, ctx->p, ctx->D);
  // H, nabla and every scalar except xi start at zero; clocks start at t_bar
  LAQ_HIP(ctx, hipMemsetAsync(ctx->ws, 0, l.xi, ctx->stream));
  LAQ_HIP(ctx, hipMemsetAsync(ctx->ws + l.srv_part, 0, l.total - l.srv_part, ctx->stream));
  hipLaunchKernelGGL(fill_i32_kernel, dim3((ctx->M + 255) / 256), dim3(256), 0, ctx->stream, ctx->sc.t,
                     ctx->t_bar, ctx->M);
  LAQ_HIP(ctx, hipGetLastError());
  return LAQ_OK;
}

int laq_create(laq_ctx** out, int32_t M, int64_t p, int32_t b, int32_t D, const float* xi,
               int32_t t_bar, float alpha, void* workspace_dev, size_t workspace_bytes,
               void* hip_stream) {
  if (!out) return LAQ_EINVAL;
  *out = nullptr;
  if (!valid_sizes(M, p, b, D) || !xi || !workspace_dev) return LAQ_EINVAL;
  if (t_bar < D || !(alpha > 0.0f) || !isfinite(alpha)) return LAQ_EINVAL;
  for (int d = 0; d < D; ++d)
    if (!(xi[d] >= 0.0f) || !isfinite(xi[d])) return LAQ_EINVAL;
  if (((uintptr_t)workspace_dev & 255) != 0) return LAQ_EINVAL;
  const Layout l = make_layout(M, p, D);
  if (workspace_bytes < l.total) return LAQ_EINVAL;

  laq_ctx* ctx = new (std::nothrow) laq_ctx();
  if (!ctx) return LAQ_EINVAL;
  ctx->M = M; ctx->p = p; ctx->b = b; ctx->D = D; ctx->t_bar = t_bar; ctx->alpha = alpha;
  ctx->p_stride = laq_p_stride(p);
  ctx->w_stride = laq_w_stride(p, b);
  int K = (63 - ceil_log2(p)) / 2;
  ctx->eps_K = K < 20 ? K : 20;
  ctx->stream = (hipStream_t)hip_stream;
  ctx->ws = (uint8_t*)workspace_dev;
  ctx->ws_bytes = workspace_bytes;
  uint8_t* w = ctx->ws;
  ctx->H = (float*)(w + l.H);
  ctx->nabla = (float*)(w + l.nabla);
  DeviceScalars& s = ctx->sc;
  s.Rpart = (uint32_t*)(w + l.Rpart);
  s.Spart = (unsigned long long*)(w + l.Spart);
  s.Npart = (unsigned long long*)(w + l.Npart);
  s.Rfin = (uint32_t*)(w + l.Rfin);
  s.Rhand = (uint32_t*)(w + l.Rhand);
  s.Sq = (long long*)(w + l.Sq);
  s.E2 = (double*)(w + l.E2);
  s.lhs = (double*)(w + l.lhs);
  s.rhs = (double*)(w + l.rhs);
  s.Ehat2 = (double*)(w + l.Ehat2);
  s.t = (int32_t*)(w + l.t);
  s.uploads = (unsigned long long*)(w + l.uploads);
  s.bits = (unsigned long long*)(w + l.bits);
  s.status = (uint32_t*)(w + l.status);
  s.srv_ticket = (uint32_t*)(w + l.srv_ticket);
  s.dtheta2 = (double*)(w + l.dtheta2);
  s.xi = (double*)(w + l.xi);
  s.srv_part = (double*)(w + l.srv_part);

  auto fail = [&](int st) { delete ctx; return st; };
  hipError_t e = hipGetDevice(&ctx->device);
  if (e != hipSuccess) return fail(LAQ_EDEVICE);
  int n_cu = 0;
  e = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, ctx->device);
  if (e != hipSuccess || n_cu <= 0) return fail(LAQ_EDEVICE);
  ctx->n_cu = n_cu;
  e = resolve_static_scratch(ctx->device, &ctx->static_scratch);   // this device is current
  if (e != hipSuccess) return fail(LAQ_EDEVICE);

  double xi64[4096];
  for (int d = 0; d < D; ++d) xi64[d] = (double)xi[d];
  int st = laq_reset(ctx);
  if (st != LAQ_OK) return fail(st);
  e = hipMemcpyAsync(s.xi, xi64, (size_t)D * 8, hipMemcpyHostToDevice, ctx->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) return fail(LAQ_EDEVICE);
  *out = ctx;
  return LAQ_OK;
}

int laq_destroy(laq_ctx* ctx) {
  if (!ctx) return LAQ_EINVAL;
  delete ctx;
  return LAQ_OK;
}

int laq_set_mode(laq_ctx* ctx, uint32_t flags) {
  if (!ctx || (flags & ~LAQ_MODE_FORCE_UPLOAD)) return LAQ_EINVAL;
  ctx->mode = flags;
  return LAQ_OK;
}

// Both entry points of the quantizer: sc says where the block partials of the passes live (the
// workspace, or this GPU's static array), sw is the grid that fits that many slots.
static int quantize_skip_impl(laq_ctx* ctx, const char* who, const float* G_dev, uint32_t* codes_dev,
                              float* R_dev, uint8_t* upload_dev, const DeviceScalars& sc, const Sweep& sw) {
  if (!G_dev || !codes_dev || !R_dev || !upload_dev)
    return set_error(ctx, LAQ_EINVAL, "%s: null pointer", who);
  if (((uintptr_t)G_dev | (uintptr_t)codes_dev) & 15)
    return set_error(ctx, LAQ_EINVAL, "%s: G_dev and codes_dev must be 16-byte aligned", who);
  QuantArgs a{};
  a.G = G_dev; a.H = ctx->H; a.codes = codes_dev; a.R_out = R_dev; a.upload = upload_dev;
  a.sc = sc;
  a.p = ctx->p; a.p_stride = ctx->p_stride; a.w_stride = ctx->w_stride;
  a.M = ctx->M; a.D = ctx->D; a.t_bar = ctx->t_bar; a.eps_K = ctx->eps_K;
  a.slots = sw.Gx;
  a.alpha = ctx->alpha; a.mode = ctx->mode;
  const dim3 grid((unsigned)sw.Gx, (unsigned)ctx->M);
  a.U = sw.U;
  a.fused_decide = sw.Gx == 1;
  if (ctx->b == LAQ_B_EXACT) {
    hipLaunchKernelGGL(exact_message_kernel, grid, dim3(kThreads), 0, ctx->stream, a);
    hipLaunchKernelGGL(exact_decide_kernel, dim3((unsigned)ctx->M), dim3(kThreads), 0, ctx->stream, a,
                       (int32_t)sw.Gx);
    LAQ_HIP(ctx, hipGetLastError());
    return LAQ_OK;
  }
  if (ctx->radius_for == G_dev && G_dev != nullptr) {
    // laq_worker_grads produced these gradients and left the block maxima of
    // |g - h| behind: the radius pass (a full read of g and h) is not needed
    a.rsrc = ctx->rprod; a.rstride = ctx->rprod_stride;
    a.rcount = ctx->rprod_count <= kDirectPartials ? ctx->rprod_count : 0;   // more: finished into Rhand when handed over
    a.rfin = ctx->sc.Rhand;
  } else {
    hipLaunchKernelGGL(radius_kernel, grid, dim3(kThreads), 0, ctx->stream, G_dev, ctx->H, ctx->p,
                       ctx->p_stride, sw.U, a.slots, sc);
    a.rsrc = sc.Rpart; a.rstride = a.slots;
    a.rcount = sw.Gx <= kDirectPartials ? sw.Gx : 0;
    a.rfin = sc.Rfin;
    if (a.rcount == 0)
      hipLaunchKernelGGL(radius_final_kernel, dim3((unsigned)ctx->M), dim3(kThreads), 0, ctx->stream,
                         sc.Rpart, a.slots, sw.Gx, sc.Rfin);
  }
#define LAQ_CALL(BB) launch_codes<BB>(grid, ctx->stream, a)
  LAQ_DISPATCH_B(ctx->b, LAQ_CALL)
#undef LAQ_CALL
  LAQ_HIP(ctx, hipGetLastError());
  return LAQ_OK;
}

int laq_quantize_skip(laq_ctx* ctx, const float* G_dev, uint32_t* codes_dev, float* R_dev,
                      uint8_t* upload_dev) {
  if (!ctx) return LAQ_EINVAL;
  return quantize_skip_impl(ctx, "laq_quantize_skip", G_dev, codes_dev, R_dev, upload_dev, ctx->sc,
                            make_sweep(ctx->p, partial_slots(ctx->M)));
}

int laq_quantize_skip_noalloc(laq_ctx* ctx, const float* G_dev, uint32_t* codes_dev, float* R_dev,
                              uint8_t* upload_dev) {
  if (!ctx) return LAQ_EINVAL;
  if (ctx->M > kStaticMaxM)
    return set_error(ctx, LAQ_EINVAL, "laq_quantize_skip_noalloc: M = %d exceeds the static scratch (at most %d workers)",
                     ctx->M, kStaticMaxM);
  if (!ctx->static_scratch)
    return set_error(ctx, LAQ_ESTATE, "laq_quantize_skip_noalloc: the static scratch of this device was not resolved");
  const Sweep sw = make_sweep(ctx->p, kStaticSlots / ctx->M);
  if (sw.U > 512)
    return set_error(ctx, LAQ_EINVAL,
                     "laq_quantize_skip_noalloc: M * p = %d * %lld exceeds the static scratch (%d block partials "
                     "of at most 512 tiles of 2048 coordinates)", ctx->M, (long long)ctx->p, kStaticSlots);
  StaticScratch* ss = reinterpret_cast<StaticScratch*>(ctx->static_scratch);
  DeviceScalars sc = ctx->sc;
  sc.Rpart = ss->Rpart; sc.Spart = ss->Spart; sc.Npart = ss->Npart; sc.Rfin = ss->Rfin;
  return quantize_skip_impl(ctx, "laq_quantize_skip_noalloc", G_dev, codes_dev, R_dev, upload_dev, sc, sw);
}

int laq_radius_handover(laq_ctx* ctx, const float* G_dev, const uint32_t* rmax_dev, int32_t count) {
  if (!ctx) return LAQ_EINVAL;
  if (count == 0) {            // withdraws a declaration (also the one laq_worker_grads leaves)
    ctx->radius_for = nullptr;
    return LAQ_OK;
  }
  if (!G_dev || !rmax_dev || count < 0)
    return set_error(ctx, LAQ_EINVAL, "laq_radius_handover: null pointer or count < 0");
  ctx->rprod = const_cast<uint32_t*>(rmax_dev);
  ctx->rprod_stride = count;
  ctx->rprod_count = count;
  if (count > kDirectPartials) {
    hipLaunchKernelGGL(radius_final_kernel, dim3((unsigned)ctx->M), dim3(kThreads), 0, ctx->stream, ctx->rprod,
                       count, count, ctx->sc.Rhand);
    LAQ_HIP(ctx, hipGetLastError());
  }
  ctx->radius_for = G_dev;
  return LAQ_OK;
}

int laq_server_step(laq_ctx* ctx, const uint32_t* codes_dev, const float* R_dev,
                    const uint8_t* upload_dev, float* theta_dev) {
  if (!ctx) return LAQ_EINVAL;
  if (!codes_dev || !R_dev || !upload_dev || !theta_dev)
    return set_error(ctx, LAQ_EINVAL, "laq_server_step: null pointer");
  if (((uintptr_t)codes_dev | (uintptr_t)theta_dev) & 15)
    return set_error(ctx, LAQ_EINVAL, "laq_server_step: codes_dev and theta_dev must be 16-byte aligned");
  ServerArgs a{};
  ctx->radius_for = nullptr;   // the stored quantized gradients change below
  a.codes = codes_dev; a.R_in = R_dev; a.upload = upload_dev;
  a.H = ctx->H; a.nabla = ctx->nabla; a.theta = theta_dev; a.sc = ctx->sc;
  a.p = ctx->p; a.p_stride = ctx->p_stride; a.w_stride = ctx->w_stride;
  a.M = ctx->M; a.D = ctx->D; a.b = ctx->b; a.alpha = ctx->alpha;
  const int64_t blocks = server_blocks(ctx->p, &a.J);
  a.fused_finish = blocks <= 32;
  const size_t smem = (size_t)(ctx->M < kServerList ? ctx->M : kServerList) * 12;
  const dim3 grid((unsigned)blocks);
#define LAQ_CALL(BB) launch_server<BB>(grid, smem, ctx->stream, a)
  if (ctx->b == LAQ_B_EXACT) LAQ_CALL(kExact);
  else LAQ_DISPATCH_B(ctx->b, LAQ_CALL)
#undef LAQ_CALL
  LAQ_HIP(ctx, hipGetLastError());
  return LAQ_OK;
}

int laq_get_state(laq_ctx* ctx, laq_state_view* v) {
  if (!ctx || !v) return LAQ_EINVAL;
  ctx->radius_for = nullptr;   // the caller may overwrite the state through these pointers
  v->H_dev = ctx->H;
  v->nabla_dev = ctx->nabla;
  v->Ehat2_dev = ctx->sc.Ehat2;
  v->t_dev = ctx->sc.t;
  v->dtheta2_dev = ctx->sc.dtheta2;
  v->Sq_dev = (int64_t*)ctx->sc.Sq;
  v->E2_dev = ctx->sc.E2;
  v->lhs_dev = ctx->sc.lhs;
  v->rhs_dev = ctx->sc.rhs;
  v->uploads_dev = (uint64_t*)ctx->sc.uploads;
  v->bits_dev = (uint64_t*)ctx->sc.bits;
  v->status_dev = ctx->sc.status;
  v->p_stride = ctx->p_stride;
  v->w_stride = ctx->w_stride;
  return LAQ_OK;
}

int laq_get_counters(laq_ctx* ctx, uint64_t* uploads, uint64_t* bits_total) {
  if (!ctx) return LAQ_EINVAL;
  uint32_t status = 0;
  if (uploads)
    LAQ_HIP(ctx, hipMemcpyAsync(uploads, ctx->sc.uploads, (size_t)ctx->M * 8, hipMemcpyDeviceToHost, ctx->stream));
  if (bits_total)
    LAQ_HIP(ctx, hipMemcpyAsync(bits_total, ctx->sc.bits, 8, hipMemcpyDeviceToHost, ctx->stream));
  LAQ_HIP(ctx, hipMemcpyAsync(&status, ctx->sc.status, 4, hipMemcpyDeviceToHost, ctx->stream));
  LAQ_HIP(ctx, hipStreamSynchronize(ctx->stream));
  if (status & 2u) return set_error(ctx, LAQ_EINVAL, "a minibatch index was outside its worker's shard");
  if (status) return set_error(ctx, LAQ_ENONFINITE, "a quantization radius was not finite");
  return LAQ_OK;
}

const char* laq_last_error(const laq_ctx* ctx) { return ctx ? ctx->err : "null context"; }

int laq_set_model(laq_ctx* ctx, int32_t kind, const int32_t* dims, int32_t n_dims, float lambda) {
  if (!ctx) return LAQ_EINVAL;
  if (!(lambda >= 0.0f) || !isfinite(lambda)) return set_error(ctx, LAQ_EINVAL, "lambda must be >= 0");
  if (kind == LAQ_MODEL_NONE) { ctx->kind = kind; return LAQ_OK; }
  if (!dims) return set_error(ctx, LAQ_EINVAL, "dims is null");
  int64_t pp = 0;
  if (kind == LAQ_MODEL_BINLOG) {
    if (n_dims != 1 || dims[0] < 1) return set_error(ctx, LAQ_EINVAL, "binary logistic: dims = {F}");
    pp = dims[0]; ctx->F = dims[0]; ctx->C = 1;
  } else if (kind == LAQ_MODEL_SOFTMAX) {
    if (n_dims != 2 || dims[0] < 1 || dims[1] < 2) return set_error(ctx, LAQ_EINVAL, "softmax: dims = {F, C}");
    pp = (int64_t)dims[0] * dims[1]; ctx->F = dims[0]; ctx->C = dims[1];
  } else if (kind == LAQ_MODEL_MLP) {
    if (n_dims < 2 || n_dims > LAQ_MAX_LAYERS + 1) return set_error(ctx, LAQ_EINVAL, "mlp: 2..%d widths", LAQ_MAX_LAYERS + 1);
    Mlp& n = ctx->mlp;
    n.n_layers = n_dims - 1;
    int64_t off = 0;
    for (int l = 0; l < n_dims; ++l) {
      if (dims[l] < 1) return set_error(ctx, LAQ_EINVAL, "mlp: widths must be >= 1");
      n.dims[l] = dims[l];
    }
    for (int l = 0; l < n.n_layers; ++l) {
      n.offW[l] = off; off += (int64_t)dims[l] * dims[l + 1];
      n.offB[l] = off; off += dims[l + 1];
    }
    pp = off; ctx->F = dims[0]; ctx->C = dims[n_dims - 1];
  } else {
    return set_error(ctx, LAQ_EINVAL, "unknown model kind %d", kind);
  }
  if (pp != ctx->p) return set_error(ctx, LAQ_EINVAL, "model has %lld parameters, context has p = %lld", (long long)pp, (long long)ctx->p);
  ctx->kind = kind;
  ctx->lambda = lambda;
  ctx->radius_for = nullptr;
  ctx->X = nullptr; ctx->y = nullptr; ctx->model_ws = nullptr;
  ctx->Xtiled = nullptr; ctx->tiled_for = nullptr; ctx->tiled_rows = 0;
  return LAQ_OK;
}

size_t laq_model_workspace_bytes(const laq_ctx* ctx, int64_t N_m) {
  if (!ctx || N_m < 1) return 0;
  return model_workspace_bytes(ctx, N_m);
}

int laq_set_data(laq_ctx* ctx, const float* X_dev, const int32_t* y_dev, int64_t N_m, int64_t ldx,
                 void* model_ws_dev, size_t model_ws_bytes) {
  if (!ctx) return LAQ_EINVAL;
  if (ctx->kind == LAQ_MODEL_NONE) return set_error(ctx, LAQ_ESTATE, "laq_set_data before laq_set_model");
  if (!X_dev || !y_dev || N_m < 1 || ldx < ctx->F || (ldx & 3) || ((uintptr_t)X_dev & 15))
    return set_error(ctx, LAQ_EINVAL, "laq_set_data: bad X/y/N_m/ldx");
  const size_t need = model_workspace_bytes(ctx, N_m);
  if (need && (!model_ws_dev || model_ws_bytes < need || ((uintptr_t)model_ws_dev & 255)))
    return set_error(ctx, LAQ_EINVAL, "laq_set_data: model workspace too small or misaligned (need %zu bytes)", need);
  ctx->X = X_dev; ctx->y = y_dev; ctx->N_m = N_m; ctx->ldx = ldx;
  ctx->model_ws = (uint8_t*)model_ws_dev; ctx->model_ws_bytes = model_ws_bytes;
  ctx->Xtiled = nullptr; ctx->tiled_for = nullptr; ctx->tiled_rows = 0;
  return LAQ_OK;
}

size_t laq_tiled_data_bytes(const laq_ctx* ctx) {
  if (!ctx || ctx->kind == LAQ_MODEL_NONE) return 0;
  return tiled_data_bytes(ctx);
}

int laq_tile_data(laq_ctx* ctx, void* tiled_dev, size_t tiled_bytes) {
  if (!ctx) return LAQ_EINVAL;
  if (ctx->kind == LAQ_MODEL_NONE || !ctx->X)
    return set_error(ctx, LAQ_ESTATE, "laq_tile_data needs laq_set_model and laq_set_data");
  const size_t need = tiled_data_bytes(ctx);
  if (need == 0) return set_error(ctx, LAQ_EINVAL, "laq_tile_data: this model has no kernel that reads tiled data");
  if (!tiled_dev || tiled_bytes < need || ((uintptr_t)tiled_dev & 255))
    return set_error(ctx, LAQ_EINVAL, "laq_tile_data: buffer too small or misaligned (need %zu bytes)", need);
  const int st = tile_data(ctx, static_cast<float*>(tiled_dev));
  if (st != LAQ_OK) return st;
  ctx->Xtiled = static_cast<const float*>(tiled_dev); ctx->tiled_for = ctx->X; ctx->tiled_rows = ctx->N_m;
  return LAQ_OK;
}

int laq_worker_grads(laq_ctx* ctx, const float* theta_dev, float* G_dev) {
  if (!ctx) return LAQ_EINVAL;
  if (ctx->kind == LAQ_MODEL_NONE || !ctx->X)
    return set_error(ctx, LAQ_ESTATE, "laq_worker_grads needs laq_set_model and laq_set_data");
  if (!theta_dev || !G_dev || (((uintptr_t)theta_dev | (uintptr_t)G_dev) & 15))
    return set_error(ctx, LAQ_EINVAL, "laq_worker_grads: null or misaligned pointer");
  ctx->radius_for = nullptr;
  const int st = worker_grads(ctx, theta_dev, G_dev);
  if (st == LAQ_OK && ctx->rprod_count > 0) {
    if (ctx->rprod_count > kDirectPartials) {
      hipLaunchKernelGGL(radius_final_kernel, dim3((unsigned)ctx->M), dim3(kThreads), 0, ctx->stream,
                         ctx->rprod, ctx->rprod_stride, ctx->rprod_count, ctx->sc.Rhand);
      LAQ_HIP(ctx, hipGetLastError());
    }
    ctx->radius_for = G_dev;
  }
  return st;
}

size_t laq_minibatch_workspace_bytes(const laq_ctx* ctx, int64_t B) {
  if (!ctx || B < 1 || ctx->kind == LAQ_MODEL_NONE || !ctx->X) return 0;
  return minibatch_layout(ctx, B).total;
}

int laq_worker_grads_minibatch(laq_ctx* ctx, const float* theta_dev, const int32_t* idx_dev, int64_t B,
                               void* ws_dev, size_t ws_bytes, float* G_dev) {
  if (!ctx) return LAQ_EINVAL;
  if (ctx->kind == LAQ_MODEL_NONE || !ctx->X)
    return set_error(ctx, LAQ_ESTATE, "laq_worker_grads_minibatch needs laq_set_model and laq_set_data");
  if (!theta_dev || !G_dev || !idx_dev || (((uintptr_t)theta_dev | (uintptr_t)G_dev) & 15))
    return set_error(ctx, LAQ_EINVAL, "laq_worker_grads_minibatch: null or misaligned pointer");
  if (B < 1 || B > ctx->N_m)
    return set_error(ctx, LAQ_EINVAL, "laq_worker_grads_minibatch: B = %lld outside 1..N_m", (long long)B);
  const MinibatchLayout l = minibatch_layout(ctx, B);
  if (!ws_dev || ws_bytes < l.total || ((uintptr_t)ws_dev & 255))
    return set_error(ctx, LAQ_EINVAL, "laq_worker_grads_minibatch: workspace too small or misaligned (need %zu bytes)",
                     l.total);
  uint8_t* ws = static_cast<uint8_t*>(ws_dev);
  const float* X0 = ctx->X; const int32_t* y0 = ctx->y; const int64_t N0 = ctx->N_m;
  uint8_t* mw0 = ctx->model_ws; const size_t mb0 = ctx->model_ws_bytes;
  if (minibatch_reads_in_place(ctx)) {
    // the gradient kernel follows the index list itself: no copy of the drawn rows
    ctx->gather_idx = idx_dev; ctx->gather_rows = N0;
  } else {
    float* Xb = reinterpret_cast<float*>(ws + l.Xb);
    int32_t* yb = reinterpret_cast<int32_t*>(ws + l.yb);
    const int64_t work = B * (ctx->ldx >> 2);
    hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)((work + kThreads - 1) / kThreads), (unsigned)ctx->M),
                       dim3(kThreads), 0, ctx->stream, ctx->X, ctx->y, idx_dev, ctx->N_m, ctx->ldx, B, Xb, yb,
                       ctx->sc.status);
    LAQ_HIP(ctx, hipGetLastError());
    ctx->X = Xb; ctx->y = yb;
  }
  // the gradient of the loss the minibatch defines: the same kernels on the drawn rows
  ctx->N_m = B;
  ctx->model_ws = ws + l.model; ctx->model_ws_bytes = l.total - l.model;
  const int st = laq_worker_grads(ctx, theta_dev, G_dev);
  ctx->X = X0; ctx->y = y0; ctx->N_m = N0; ctx->model_ws = mw0; ctx->model_ws_bytes = mb0;
  ctx->gather_idx = nullptr; ctx->gather_rows = 0;
  return st;
}

}  // extern "C"
