// Internal declarations shared by the translation units of liblaq_hip.so.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "laq.h"

namespace laq {

constexpr int kThreads = 256;          // 4 wavefronts of 64 lanes
constexpr int kGroup = 8;              // elements owned by one lane per step: 8*b bits = b whole bytes

// Per-worker and global scalars kept in the device workspace.
struct DeviceScalars {
  uint32_t* Rpart;              // [M][slots] block maxima of |g-h| (raw bits)
  unsigned long long* Spart;    // [M][slots] block sums of (2q-L)^2
  unsigned long long* Npart;    // [M][slots] block sums of the integer error squares
  uint32_t* Rfin;               // [M] radius found by the current call's own radius pass (raw bits)
  uint32_t* Rhand;              // [M] radius finished from a producer's block maxima (hand-over); never
                                //     written by a radius pass, so it stays valid as long as the hand-over does
  long long* Sq;                // [M] stash
  double* E2;                   // [M] stash
  double* lhs;                  // [M]
  double* rhs;                  // [M]
  double* Ehat2;                // [M]
  int32_t* t;                   // [M]
  unsigned long long* uploads;  // [M]
  unsigned long long* bits;     // [1]
  uint32_t* status;             // [1]
  uint32_t* srv_ticket;         // [1]
  double* dtheta2;              // [D]
  double* xi;                   // [D]
  double* srv_part;             // [server blocks] partial sums of ||nabla||^2
};

struct Mlp {
  int32_t n_layers = 0;                 // weight layers
  int32_t dims[LAQ_MAX_LAYERS + 1] = {0};
  int64_t offW[LAQ_MAX_LAYERS] = {0};
  int64_t offB[LAQ_MAX_LAYERS] = {0};
};

}  // namespace laq

struct laq_ctx {
  int32_t M = 0;
  int64_t p = 0, p_stride = 0, w_stride = 0;
  int32_t b = 0, D = 0, t_bar = 0, eps_K = 0;
  float alpha = 0.f;
  uint32_t mode = 0;
  hipStream_t stream = nullptr;
  int device = 0;
  int n_cu = 256;

  uint8_t* ws = nullptr;
  size_t ws_bytes = 0;
  float* H = nullptr;
  float* nabla = nullptr;
  laq::DeviceScalars sc{};
  size_t scalars_offset = 0, scalars_bytes = 0;
  // device address of this GPU's static scratch array (laq_quantize_skip_noalloc), resolved by laq_create
  unsigned char* static_scratch = nullptr;

  // Radius hand-over from laq_worker_grads to laq_quantize_skip: the gradient
  // kernels' epilogues leave block maxima of |g - h| in rprod[m][0..rprod_count);
  // valid only for the G pointer in radius_for and until the state changes.
  const float* radius_for = nullptr;
  // Minibatch call in flight: the matrix-core softmax kernel reads the drawn rows through this
  // index list [M][N_m] from shards of gather_rows rows (else nullptr).
  const int32_t* gather_idx = nullptr;
  int64_t gather_rows = 0;
  uint32_t* rprod = nullptr;
  int32_t rprod_stride = 0, rprod_count = 0;

  // model
  int32_t kind = LAQ_MODEL_NONE;
  float lambda = 0.f;
  int32_t F = 0, C = 0;
  laq::Mlp mlp{};
  const float* X = nullptr;
  const int32_t* y = nullptr;
  int64_t N_m = 0, ldx = 0;
  // Tiled copy of X made by laq_tile_data (caller-owned memory): stands for tiled_for[M][tiled_rows].
  const float* Xtiled = nullptr;
  const float* tiled_for = nullptr;
  int64_t tiled_rows = 0;
  uint8_t* model_ws = nullptr;
  size_t model_ws_bytes = 0;

  char err[512] = {0};
};

namespace laq {

int set_error(laq_ctx* ctx, int status, const char* fmt, ...);

#define LAQ_HIP(ctx, expr)                                                          \
  do {                                                                              \
    hipError_t _e = (expr);                                                         \
    if (_e != hipSuccess)                                                           \
      return laq::set_error((ctx), LAQ_EDEVICE, "%s failed: %s (%s:%d)", #expr,     \
                            hipGetErrorString(_e), __FILE__, __LINE__);             \
  } while (0)

// gradient kernels (laq_grads.hip)
size_t model_workspace_bytes(const laq_ctx* ctx, int64_t N_m);
int worker_grads(laq_ctx* ctx, const float* theta, float* G);
bool minibatch_reads_in_place(const laq_ctx* ctx);
size_t tiled_data_bytes(const laq_ctx* ctx);
int tile_data(laq_ctx* ctx, float* Xt);

}  // namespace laq
