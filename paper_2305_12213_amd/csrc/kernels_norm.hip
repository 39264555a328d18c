// Batch normalisation over each worker's own rows and residual additions (bf16 storage).
// A "row" is a sample or a pixel; worker k owns rows [off_k, off_{k+1}).  The statistics of
// a worker never see another worker's rows, so every reduction here runs per (worker, channel):
// one workgroup takes 64 channels of one worker, 4 row-lanes per channel, rows read as 128
// contiguous bytes.  All sums are fp32 in a fixed order (deterministic).
#include <hip/hip_runtime.h>

#include "dynb_internal.h"

namespace dynb {
namespace {

typedef __bf16 bf16;

__device__ inline int worker_of_row(const Segs& s, int row) {
  int k = 0;
  while (k + 1 < s.K && row >= s.off[k + 1]) ++k;
  return k;
}

// Sum over the 4 row-lanes of a channel: threads are laid out [row-lane][channel], the partial
// sums meet in LDS and every thread of the channel reads the total (fixed order 0..3).
__device__ inline float sum4(float v, float (*red)[64], int rl, int cl) {
  __syncthreads();
  red[rl][cl] = v;
  __syncthreads();
  return ((red[0][cl] + red[1][cl]) + red[2][cl]) + red[3][cl];
}

// mean[k][c], rstd[k][c] of x over worker k's rows: two passes (mean, then centred squares).
__global__ __launch_bounds__(256) void bn_stats_kernel(const bf16* __restrict__ x, int64_t ld, int C,
                                                       float eps, float* __restrict__ mean,
                                                       float* __restrict__ rstd, Segs s) {
  __shared__ float red[4][64];
  const int cl = threadIdx.x & 63, rl = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + cl, k = blockIdx.y;
  const int r0 = s.off[k], n = s.off[k + 1] - r0;
  if (n <= 0) return;                         // (uniform over the workgroup)
  const bool live = c < C;
  float acc = 0.f;
  if (live)
    for (int r = rl; r < n; r += 4) acc += (float)x[(int64_t)(r0 + r) * ld + c];
  const float mu = sum4(acc, red, rl, cl) / (float)n;
  acc = 0.f;
  if (live)
    for (int r = rl; r < n; r += 4) {
      const float d = (float)x[(int64_t)(r0 + r) * ld + c] - mu;
      acc += d * d;
    }
  const float var = sum4(acc, red, rl, cl) / (float)n;
  if (live && rl == 0) {
    mean[(int64_t)k * C + c] = mu;
    rstd[(int64_t)k * C + c] = 1.f / sqrtf(var + eps);
  }
}

// y = relu?(gamma * (x - mean_k) * rstd_k + beta)
__global__ __launch_bounds__(256) void bn_forward_kernel(const bf16* __restrict__ x, int64_t ldx,
                                                         int C, const float* __restrict__ gamma,
                                                         const float* __restrict__ beta,
                                                         const float* __restrict__ mean,
                                                         const float* __restrict__ rstd, int relu,
                                                         bf16* __restrict__ y, int64_t ldy, Segs s) {
  const int c = blockIdx.x * 256 + threadIdx.x, row = blockIdx.y;
  if (c >= C) return;
  const int k = worker_of_row(s, row);
  const float xh = ((float)x[(int64_t)row * ldx + c] - mean[(int64_t)k * C + c]) * rstd[(int64_t)k * C + c];
  float v = gamma[c] * xh + beta[c];
  if (relu) v = fmaxf(v, 0.f);
  y[(int64_t)row * ldy + c] = (bf16)v;
}

// dgamma[k][c] = sum_rows dy * xhat, dbeta[k][c] = sum_rows dy  (dy already carries this
// layer's ReLU mask) -> worker k's gradient vector
__global__ __launch_bounds__(256) void bn_param_grad_kernel(const bf16* __restrict__ dy, int64_t ldd,
                                                            const bf16* __restrict__ x, int64_t ldx,
                                                            int C, const float* __restrict__ mean,
                                                            const float* __restrict__ rstd,
                                                            float* __restrict__ dgamma,
                                                            float* __restrict__ dbeta,
                                                            int64_t group_stride, Segs s) {
  __shared__ float red[4][64];
  const int cl = threadIdx.x & 63, rl = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + cl, k = blockIdx.y;
  const int r0 = s.off[k], n = s.off[k + 1] - r0;
  const bool live = c < C;
  float ag = 0.f, ab = 0.f;
  if (live && n > 0) {
    const float mu = mean[(int64_t)k * C + c], rs = rstd[(int64_t)k * C + c];
    for (int r = rl; r < n; r += 4) {
      const float d = (float)dy[(int64_t)(r0 + r) * ldd + c];
      ab += d;
      ag += d * (((float)x[(int64_t)(r0 + r) * ldx + c] - mu) * rs);
    }
  }
  const float tg = sum4(ag, red, rl, cl);
  const float tb = sum4(ab, red, rl, cl);
  if (live && rl == 0) {                      // an idle worker gets zeros
    dgamma[(int64_t)k * group_stride + c] = tg;
    dbeta[(int64_t)k * group_stride + c] = tb;
  }
}

// dx = gamma * rstd * (dy - dbeta/n - xhat * dgamma/n), masked by the producer's ReLU
__global__ __launch_bounds__(256) void bn_input_grad_kernel(
    const bf16* __restrict__ dy, int64_t ldd, const bf16* __restrict__ x, int64_t ldx, int C,
    const float* __restrict__ gamma, const float* __restrict__ mean, const float* __restrict__ rstd,
    const float* __restrict__ dgamma, const float* __restrict__ dbeta, int64_t group_stride,
    int relu_below, bf16* __restrict__ dx, int64_t ldo, Segs s) {
  const int c = blockIdx.x * 256 + threadIdx.x, row = blockIdx.y;
  if (c >= C) return;
  const int k = worker_of_row(s, row);
  const float n = (float)(s.off[k + 1] - s.off[k]);
  const float xv = (float)x[(int64_t)row * ldx + c];
  const float rs = rstd[(int64_t)k * C + c];
  const float xh = (xv - mean[(int64_t)k * C + c]) * rs;
  float v = gamma[c] * rs * ((float)dy[(int64_t)row * ldd + c] - dbeta[(int64_t)k * group_stride + c] / n -
                             xh * (dgamma[(int64_t)k * group_stride + c] / n));
  if (relu_below && !(xv > 0.f)) v = 0.f;
  dx[(int64_t)row * ldo + c] = (bf16)v;
}

// out = relu?(a + b)
__global__ __launch_bounds__(256) void add_forward_kernel(const bf16* __restrict__ a, int64_t lda,
                                                          const bf16* __restrict__ b, int64_t ldb,
                                                          int C, int relu, bf16* __restrict__ out,
                                                          int64_t ldo) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  const int64_t row = blockIdx.y;
  if (c >= C) return;
  float v = (float)a[row * lda + c] + (float)b[row * ldb + c];
  if (relu) v = fmaxf(v, 0.f);
  out[row * ldo + c] = (bf16)v;
}

// dst = (accumulate ? dst : 0) + src, masked by act > 0 when `relu` (act = the stored output of
// the layer whose gradient dst is)
__global__ __launch_bounds__(256) void grad_route_kernel(const bf16* __restrict__ src, int64_t lds_,
                                                         const bf16* __restrict__ act, int64_t lda,
                                                         int C, int relu, int accumulate,
                                                         bf16* __restrict__ dst, int64_t ldd) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  const int64_t row = blockIdx.y;
  if (c >= C) return;
  float v = (float)src[row * lds_ + c];
  if (relu && !((float)act[row * lda + c] > 0.f)) v = 0.f;
  if (accumulate) v += (float)dst[row * ldd + c];
  dst[row * ldd + c] = (bf16)v;
}

inline int ok(const char* what) {
  return hipGetLastError() == hipSuccess ? DYNB_OK : fail(DYNB_ERR_HIP, "%s: launch failed", what);
}

}  // namespace

int launch_bn_forward(const void* x, int64_t ldx, int C, const float* gamma, const float* beta,
                      float eps, int relu, float* mean, float* rstd, void* y, int64_t ldy,
                      const Segs& s, void* stream) {
  const int rows = s.off[s.K];
  if (rows == 0 || C == 0) return DYNB_OK;
  Timed t(KC_CONV_AUX, stream, 0, (double)rows * C * 8);
  hipLaunchKernelGGL(bn_stats_kernel, dim3((C + 63) / 64, s.K), dim3(256), 0, (hipStream_t)stream,
                     (const bf16*)x, ldx, C, eps, mean, rstd, s);
  hipLaunchKernelGGL(bn_forward_kernel, dim3((C + 255) / 256, rows), dim3(256), 0, (hipStream_t)stream,
                     (const bf16*)x, ldx, C, gamma, beta, mean, rstd, relu, (bf16*)y, ldy, s);
  return ok("bn_forward");
}

int launch_bn_backward(const void* dy, int64_t ldd, const void* x, int64_t ldx, int C,
                       const float* gamma, const float* mean, const float* rstd, float* dgamma,
                       float* dbeta, int64_t group_stride, int need_dx, int relu_below, void* dx,
                       int64_t ldo, const Segs& s, void* stream) {
  const int rows = s.off[s.K];
  if (C == 0) return DYNB_OK;
  Timed t(KC_CONV_AUX, stream, 0, (double)rows * C * 10);
  hipLaunchKernelGGL(bn_param_grad_kernel, dim3((C + 63) / 64, s.K), dim3(256), 0, (hipStream_t)stream,
                     (const bf16*)dy, ldd, (const bf16*)x, ldx, C, mean, rstd, dgamma, dbeta,
                     group_stride, s);
  if (need_dx && rows > 0)
    hipLaunchKernelGGL(bn_input_grad_kernel, dim3((C + 255) / 256, rows), dim3(256), 0,
                       (hipStream_t)stream, (const bf16*)dy, ldd, (const bf16*)x, ldx, C, gamma, mean,
                       rstd, dgamma, dbeta, group_stride, relu_below, (bf16*)dx, ldo, s);
  return ok("bn_backward");
}

int launch_add_forward(const void* a, int64_t lda, const void* b, int64_t ldb, int C, int64_t rows,
                       int relu, void* out, int64_t ldo, void* stream) {
  if (rows == 0 || C == 0) return DYNB_OK;
  Timed t(KC_CONV_AUX, stream, 0, (double)rows * C * 6);
  hipLaunchKernelGGL(add_forward_kernel, dim3((C + 255) / 256, (unsigned)rows), dim3(256), 0,
                     (hipStream_t)stream, (const bf16*)a, lda, (const bf16*)b, ldb, C, relu,
                     (bf16*)out, ldo);
  return ok("add_forward");
}

int launch_grad_route(const void* src, int64_t lds_, const void* act, int64_t lda, int C,
                      int64_t rows, int relu, int accumulate, void* dst, int64_t ldd, void* stream) {
  if (rows == 0 || C == 0) return DYNB_OK;
  Timed t(KC_CONV_AUX, stream, 0, (double)rows * C * 6);
  hipLaunchKernelGGL(grad_route_kernel, dim3((C + 255) / 256, (unsigned)rows), dim3(256), 0,
                     (hipStream_t)stream, (const bf16*)src, lds_, (const bf16*)act, lda, C, relu,
                     accumulate, (bf16*)dst, ldd);
  return ok("grad_route");
}

}  // namespace dynb
