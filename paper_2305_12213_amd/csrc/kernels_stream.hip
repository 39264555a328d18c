// HBM-streaming kernels: weighted aggregation (Eq. 2), SGD / momentum update (Eq. 3).
// One 16-byte access per lane and array; grid-stride over float4 elements.
#include <hip/hip_runtime.h>

#include "dynb_internal.h"

namespace dynb {
namespace {

constexpr int kThreads = 256;
typedef float f4 __attribute__((ext_vector_type(4)));

// out[p] = sum_k w_k * grads[k][p], k ascending.  Loads of UNROLL workers are issued
// before they are consumed so that several 16-byte reads per lane are in flight.
template <int UNROLL>
__global__ __launch_bounds__(kThreads) void aggregate_kernel(const f4* __restrict__ grads,
                                                             int64_t stride4, Lambdas lam,
                                                             int64_t n4, f4* __restrict__ out) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n4; i += stride) {
    f4 acc = {0.f, 0.f, 0.f, 0.f};
    int k = 0;
    for (; k + UNROLL <= lam.K; k += UNROLL) {
      f4 v[UNROLL];
#pragma unroll
      for (int u = 0; u < UNROLL; ++u)
        v[u] = __builtin_nontemporal_load(&grads[(int64_t)(k + u) * stride4 + i]);
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) {
        acc += lam.w[k + u] * v[u];
      }
    }
    for (; k < lam.K; ++k) {
      const f4 v = __builtin_nontemporal_load(&grads[(int64_t)k * stride4 + i]);
      acc += lam.w[k] * v;
    }
    out[i] = acc;
  }
}

// The same sum over a range of any alignment (biases, small weights): one element per lane.
__global__ __launch_bounds__(kThreads) void aggregate_range_kernel(const float* __restrict__ g,
                                                                   int64_t worker_stride,
                                                                   Lambdas lam, int64_t n,
                                                                   float* __restrict__ out) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) {
    float acc = 0.f;
    for (int k = 0; k < lam.K; ++k) acc += lam.w[k] * g[(int64_t)k * worker_stride + i];
    out[i] = acc;
  }
}

// ... and over a list of such ranges (blockIdx.y = range)
__global__ __launch_bounds__(kThreads) void aggregate_ranges_kernel(const float* __restrict__ g,
                                                                    int64_t worker_stride,
                                                                    Lambdas lam, Ranges r,
                                                                    float* __restrict__ out) {
  const int64_t off = r.off[blockIdx.y], n = r.len[blockIdx.y];
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) {
    float acc = 0.f;
    for (int k = 0; k < lam.K; ++k) acc += lam.w[k] * g[(int64_t)k * worker_stride + off + i];
    out[off + i] = acc;
  }
}

__global__ __launch_bounds__(kThreads) void sgd_kernel(float4* __restrict__ x,
                                                       const float4* __restrict__ g, int64_t n4,
                                                       float lr) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n4; i += stride) {
    float4 p = x[i];
    const float4 d = g[i];
    p.x -= lr * d.x;
    p.y -= lr * d.y;
    p.z -= lr * d.z;
    p.w -= lr * d.w;
    x[i] = p;
  }
}

__global__ __launch_bounds__(kThreads) void momentum_kernel(float4* __restrict__ x,
                                                            float4* __restrict__ vel,
                                                            const float4* __restrict__ g,
                                                            int64_t n4, float lr, float mu) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n4; i += stride) {
    float4 p = x[i];
    float4 v = vel[i];
    const float4 d = g[i];
    v.x = mu * v.x + d.x;
    v.y = mu * v.y + d.y;
    v.z = mu * v.z + d.z;
    v.w = mu * v.w + d.w;
    p.x -= lr * v.x;
    p.y -= lr * v.y;
    p.z -= lr * v.z;
    p.w -= lr * v.w;
    vel[i] = v;
    x[i] = p;
  }
}

int grid_for(int64_t n4) {
  int64_t blocks = (n4 + kThreads - 1) / kThreads;
  const int64_t cap = 256 * 16;  // 16 workgroups per compute unit
  if (blocks > cap) blocks = cap;
  if (blocks < 1) blocks = 1;
  return (int)blocks;
}

}  // namespace

int launch_aggregate(const float* grads, const Lambdas& lam, int64_t n, float* out, void* stream) {
  const int64_t n4 = n / 4;
  if (n4 == 0) return DYNB_OK;
  Timed t(KC_AGGREGATE, stream, 2.0 * lam.K * n, 4.0 * (lam.K + 1) * n);
  hipLaunchKernelGGL(aggregate_kernel<4>, dim3(grid_for(n4)), dim3(kThreads), 0,
                     (hipStream_t)stream, (const f4*)grads, n4, lam, n4, (f4*)out);
  return hipGetLastError() == hipSuccess ? DYNB_OK : fail(DYNB_ERR_HIP, "aggregate launch failed");
}

int launch_aggregate_range(const float* g, int64_t worker_stride, const Lambdas& lam, int64_t n,
                           float* out, void* stream) {
  if (n <= 0) return DYNB_OK;
  Timed t(KC_AGGREGATE, stream, 2.0 * lam.K * n, 4.0 * (lam.K + 1) * n);
  if (n >= 4096 && !(n & 3) && !(worker_stride & 3) && !(((uintptr_t)g | (uintptr_t)out) & 15)) {
    hipLaunchKernelGGL(aggregate_kernel<4>, dim3(grid_for(n / 4)), dim3(kThreads), 0,
                       (hipStream_t)stream, (const f4*)g, worker_stride / 4, lam, n / 4, (f4*)out);
    return hipGetLastError() == hipSuccess ? DYNB_OK : fail(DYNB_ERR_HIP, "aggregate launch failed");
  }
  int64_t blocks = (n + kThreads - 1) / kThreads;
  if (blocks > 256 * 16) blocks = 256 * 16;
  hipLaunchKernelGGL(aggregate_range_kernel, dim3((unsigned)blocks), dim3(kThreads), 0,
                     (hipStream_t)stream, g, worker_stride, lam, n, out);
  return hipGetLastError() == hipSuccess ? DYNB_OK : fail(DYNB_ERR_HIP, "aggregate launch failed");
}

int launch_aggregate_ranges(const float* g, int64_t worker_stride, const Lambdas& lam,
                            const Ranges& r, float* out, void* stream) {
  int64_t longest = 0, total = 0;
  for (int i = 0; i < r.n; ++i) {
    longest = r.len[i] > longest ? r.len[i] : longest;
    total += r.len[i];
  }
  if (r.n <= 0 || longest <= 0) return DYNB_OK;
  Timed t(KC_AGGREGATE, stream, 2.0 * lam.K * total, 4.0 * (lam.K + 1) * total);
  int64_t bx = (longest + kThreads - 1) / kThreads;
  if (bx > 1024) bx = 1024;
  hipLaunchKernelGGL(aggregate_ranges_kernel, dim3((unsigned)bx, r.n), dim3(kThreads), 0,
                     (hipStream_t)stream, g, worker_stride, lam, r, out);
  return hipGetLastError() == hipSuccess ? DYNB_OK : fail(DYNB_ERR_HIP, "aggregate launch failed");
}

int launch_sgd(float* params, const float* g, int64_t n, float lr, void* stream) {
  const int64_t n4 = n / 4;
  if (n4 == 0) return DYNB_OK;
  Timed t(KC_UPDATE, stream, 2.0 * n, 12.0 * n);
  hipLaunchKernelGGL(sgd_kernel, dim3(grid_for(n4)), dim3(kThreads), 0, (hipStream_t)stream,
                     (float4*)params, (const float4*)g, n4, lr);
  return hipGetLastError() == hipSuccess ? DYNB_OK : fail(DYNB_ERR_HIP, "sgd launch failed");
}

int launch_momentum(float* params, float* v, const float* g, int64_t n, float lr, float mu,
                    void* stream) {
  const int64_t n4 = n / 4;
  if (n4 == 0) return DYNB_OK;
  Timed t(KC_UPDATE, stream, 4.0 * n, 20.0 * n);
  hipLaunchKernelGGL(momentum_kernel, dim3(grid_for(n4)), dim3(kThreads), 0, (hipStream_t)stream,
                     (float4*)params, (float4*)v, (const float4*)g, n4, lr, mu);
  return hipGetLastError() == hipSuccess ? DYNB_OK : fail(DYNB_ERR_HIP, "momentum launch failed");
}

}  // namespace dynb

using namespace dynb;

extern "C" int dynb_weighted_aggregate(const float* grads, const int32_t* b, int32_t K, int64_t n,
                                       float* out, void* stream) {
  if (!grads || !b || !out) return fail(DYNB_ERR_BADARG, "aggregate: null pointer");
  if (K < 1 || K > DYNB_MAX_WORKERS) return fail(DYNB_ERR_BADARG, "aggregate: K out of range");
  if (n < 0 || (n & 3)) return fail(DYNB_ERR_BADARG, "aggregate: n must be a non-negative multiple of 4");
  if (((uintptr_t)grads | (uintptr_t)out) & 15)
    return fail(DYNB_ERR_BADARG, "aggregate: pointers must be 16-byte aligned");
  int64_t total = 0;
  for (int k = 0; k < K; ++k) {
    if (b[k] < 0) return fail(DYNB_ERR_BADARG, "aggregate: negative batch size");
    total += b[k];
  }
  if (total <= 0) return fail(DYNB_ERR_BADARG, "aggregate: sum(b) must be positive");
  Lambdas lam;
  lam.K = K;
  for (int k = 0; k < K; ++k) lam.w[k] = (float)((double)b[k] / (double)total);
  return launch_aggregate(grads, lam, n, out, stream);
}

extern "C" int dynb_sgd_update(float* params, const float* g, int64_t n, float lr, void* stream) {
  if (!params || !g) return fail(DYNB_ERR_BADARG, "sgd: null pointer");
  if (n < 0 || (n & 3)) return fail(DYNB_ERR_BADARG, "sgd: n must be a non-negative multiple of 4");
  if (((uintptr_t)params | (uintptr_t)g) & 15)
    return fail(DYNB_ERR_BADARG, "sgd: pointers must be 16-byte aligned");
  return launch_sgd(params, g, n, lr, stream);
}

extern "C" int dynb_sgd_momentum_update(float* params, float* velocity, const float* g, int64_t n,
                                        float lr, float mu, void* stream) {
  if (!params || !g || !velocity) return fail(DYNB_ERR_BADARG, "momentum: null pointer");
  if (n < 0 || (n & 3)) return fail(DYNB_ERR_BADARG, "momentum: n must be a non-negative multiple of 4");
  if (((uintptr_t)params | (uintptr_t)g | (uintptr_t)velocity) & 15)
    return fail(DYNB_ERR_BADARG, "momentum: pointers must be 16-byte aligned");
  return launch_momentum(params, velocity, g, n, lr, mu, stream);
}
