// Optimizer steps on the flat fp32 parameter vector: plain SGD (Eq. 3), heavy-ball momentum and
// Adam (the optimizers of the paper's workloads), optionally with the weighted aggregation of
// Eq. 2 folded in (the K per-worker gradients are read and summed where the step is applied, so
// the aggregate never goes through HBM), and fused with the refresh of the 16-bit weight copies.
#include <hip/hip_runtime.h>

#include <cmath>

#include "dynb_internal.h"

namespace dynb {
namespace {

typedef __bf16 bf16;
typedef float f4 __attribute__((ext_vector_type(4)));

template <typename T> __device__ inline T from_float(float v) { return (T)v; }

// One parameter, one step.  s1/s2 are the optimizer's state for this parameter.
template <int KIND>
__device__ inline float step_one(const UpdateRule& r, float w, float g, float& s1, float& s2) {
  if (KIND == DYNB_OPT_SGD) return w - r.lr * g;
  if (KIND == DYNB_OPT_MOMENTUM) {
    s1 = r.mu * s1 + g;
    return w - r.lr * s1;
  }
  s1 = r.beta1 * s1 + r.omb1 * g;
  s2 = r.beta2 * s2 + r.omb2 * g * g;
  return w - r.lr * (s1 * r.inv_c1) / (sqrtf(s2 * r.inv_c2) + r.eps);
}

// Gradient of 4 consecutive parameters starting at o (16-byte aligned).
template <bool AGG>
__device__ inline f4 gradient4(const GradSource& src, int64_t o) {
  if (!AGG) return *(const f4*)(src.g + o);
  constexpr int U = 8;   // loads in flight per lane
  f4 acc = {0.f, 0.f, 0.f, 0.f};
  int k = 0;
  for (; k + U <= src.lam.K; k += U) {
    f4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u)
      v[u] = __builtin_nontemporal_load((const f4*)(src.g + (int64_t)(k + u) * src.worker_stride + o));
#pragma unroll
    for (int u = 0; u < U; ++u) acc += src.lam.w[k + u] * v[u];
  }
  for (; k < src.lam.K; ++k)
    acc += src.lam.w[k] *
           __builtin_nontemporal_load((const f4*)(src.g + (int64_t)k * src.worker_stride + o));
  return acc;
}
template <bool AGG>
__device__ inline float gradient1(const GradSource& src, int64_t o) {
  if (!AGG) return src.g[o];
  float acc = 0.f;
  for (int k = 0; k < src.lam.K; ++k) acc += src.lam.w[k] * src.g[(int64_t)k * src.worker_stride + o];
  return acc;
}

// ---- dense weight matrices: step + both 16-bit copies in one pass ---------------------------
// W[r][c] <- step(W[r][c]); Wn[r][c] = T(W), Wt[c][r] = T(W).  A workgroup owns a 64 x TC tile:
// 16-byte accesses on the fp32 side, the transposed copy goes through an LDS tile so that its
// stores are 16 bytes per lane and whole 128-byte lines per 8 (bf16) lanes.
// One launch serves every matrix of `mats` (workgroups mats.first_block[i] ... belong to matrix
// i) and, with the workgroups behind the last tile, the small tensors of `small` (biases):
// back-to-back launches on one stream leave the chip idle for a few microseconds each, which
// for a four-layer model came to a sixth of the whole update.
template <typename T, int KIND, bool AGG, int TC>
__global__ __launch_bounds__(256) void update_cast_kernel(float* __restrict__ params, CastMats mats,
                                                          Ranges small, int range_blocks,
                                                          GradSource src, UpdateRule rule,
                                                          float* __restrict__ s1,
                                                          float* __restrict__ s2) {
  const int blk = blockIdx.x;
  if (blk >= mats.first_block[mats.n]) {   // the small tensors, element by element
    const int rb = blk - mats.first_block[mats.n];
    for (int q = 0; q < small.n; ++q) {
      const int64_t off = small.off[q], n = small.len[q];
      for (int64_t i = (int64_t)rb * 256 + threadIdx.x; i < n; i += (int64_t)range_blocks * 256) {
        const int64_t o = off + i;
        float a = KIND != DYNB_OPT_SGD ? s1[o] : 0.f;
        float b = KIND == DYNB_OPT_ADAM ? s2[o] : 0.f;
        params[o] = step_one<KIND>(rule, params[o], gradient1<AGG>(src, o), a, b);
        if (KIND != DYNB_OPT_SGD) s1[o] = a;
        if (KIND == DYNB_OPT_ADAM) s2[o] = b;
      }
    }
    return;
  }
  int mi = 0;
  while (blk >= mats.first_block[mi + 1]) ++mi;
  const int64_t off = mats.off[mi], ldn = mats.ldn[mi], ldt = mats.ldt[mi];
  const int R = mats.R[mi], C = mats.C[mi];
  T* __restrict__ Wn = (T*)mats.Wn[mi];
  T* __restrict__ Wt = (T*)mats.Wt[mi];
  const int tiles_x = (C + TC - 1) / TC, local = blk - mats.first_block[mi];
  const int tile_x = local % tiles_x, tile_y = local / tiles_x;
  constexpr int G = 16 / sizeof(T);
  typedef T vecT __attribute__((ext_vector_type(G)));
  typedef T vec4T __attribute__((ext_vector_type(4)));
  constexpr int QC = TC / 4;   // 16-byte granules per tile row
  __shared__ float tile[64][TC + 1];
  const int r0 = tile_y * 64, c0 = tile_x * TC;
  // 16-byte accesses need aligned rows in every array (all start at a multiple of 4 floats)
  const bool vec = (C & 3) == 0 && (off & 3) == 0;
#pragma unroll 2
  for (int idx = threadIdx.x; idx < 64 * QC; idx += 256) {
    const int r = idx / QC, cq = (idx % QC) * 4;
    const int gr = r0 + r, gc = c0 + cq;
    f4 w = {0.f, 0.f, 0.f, 0.f};
    if (gr < R && gc < C) {
      const int64_t o = off + (int64_t)gr * C + gc;
      if (vec) {
        const f4 d = gradient4<AGG>(src, o);
        w = *(const f4*)(params + o);
        f4 a = {0.f, 0.f, 0.f, 0.f}, b = a;
        if (KIND != DYNB_OPT_SGD) a = *(const f4*)(s1 + o);
        if (KIND == DYNB_OPT_ADAM) b = *(const f4*)(s2 + o);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float ae = a[e], be = b[e];
          w[e] = step_one<KIND>(rule, w[e], d[e], ae, be);
          a[e] = ae;
          b[e] = be;
        }
        *(f4*)(params + o) = w;
        if (KIND != DYNB_OPT_SGD) *(f4*)(s1 + o) = a;
        if (KIND == DYNB_OPT_ADAM) *(f4*)(s2 + o) = b;
        const vec4T q = {from_float<T>(w[0]), from_float<T>(w[1]), from_float<T>(w[2]), from_float<T>(w[3])};
        *(vec4T*)(Wn + (int64_t)gr * ldn + gc) = q;
      } else {
        for (int e = 0; e < 4 && gc + e < C; ++e) {
          float ae = KIND != DYNB_OPT_SGD ? s1[o + e] : 0.f;
          float be = KIND == DYNB_OPT_ADAM ? s2[o + e] : 0.f;
          w[e] = step_one<KIND>(rule, params[o + e], gradient1<AGG>(src, o + e), ae, be);
          params[o + e] = w[e];
          if (KIND != DYNB_OPT_SGD) s1[o + e] = ae;
          if (KIND == DYNB_OPT_ADAM) s2[o + e] = be;
          Wn[(int64_t)gr * ldn + gc + e] = from_float<T>(w[e]);
        }
      }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) tile[r][cq + e] = w[e];
  }
  __syncthreads();
  constexpr int GR = 64 / G;   // granules of rows per tile column
  for (int idx = threadIdx.x; idx < TC * GR; idx += 256) {
    const int rg = idx % GR, c = idx / GR;
    if (c0 + c >= C) continue;
    if (r0 + rg * G + G <= R) {
      vecT v;
#pragma unroll
      for (int e = 0; e < G; ++e) v[e] = from_float<T>(tile[rg * G + e][c]);
      *(vecT*)(Wt + (int64_t)(c0 + c) * ldt + r0 + rg * G) = v;
    } else {
      for (int e = 0; e < G && r0 + rg * G + e < R; ++e)
        Wt[(int64_t)(c0 + c) * ldt + r0 + rg * G + e] = from_float<T>(tile[rg * G + e][c]);
    }
  }
}

// ---- element-wise step of params[off, off + n) (biases, convolution weights) ---------------
template <int KIND, bool AGG>
__global__ __launch_bounds__(256) void update_range_kernel(float* __restrict__ params, int64_t off,
                                                           GradSource src, UpdateRule rule,
                                                           float* __restrict__ s1,
                                                           float* __restrict__ s2, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int64_t o = off + i;
    float a = KIND != DYNB_OPT_SGD ? s1[o] : 0.f;
    float b = KIND == DYNB_OPT_ADAM ? s2[o] : 0.f;
    params[o] = step_one<KIND>(rule, params[o], gradient1<AGG>(src, o), a, b);
    if (KIND != DYNB_OPT_SGD) s1[o] = a;
    if (KIND == DYNB_OPT_ADAM) s2[o] = b;
  }
}

// the same over a list of ranges (blockIdx.y = range)
template <int KIND, bool AGG>
__global__ __launch_bounds__(256) void update_ranges_kernel(float* __restrict__ params, Ranges r,
                                                            GradSource src, UpdateRule rule,
                                                            float* __restrict__ s1,
                                                            float* __restrict__ s2) {
  const int64_t off = r.off[blockIdx.y], n = r.len[blockIdx.y];
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int64_t o = off + i;
    float a = KIND != DYNB_OPT_SGD ? s1[o] : 0.f;
    float b = KIND == DYNB_OPT_ADAM ? s2[o] : 0.f;
    params[o] = step_one<KIND>(rule, params[o], gradient1<AGG>(src, o), a, b);
    if (KIND != DYNB_OPT_SGD) s1[o] = a;
    if (KIND == DYNB_OPT_ADAM) s2[o] = b;
  }
}

// ---- plain streaming Adam ----------------------------------------------------------------------
__global__ __launch_bounds__(256) void adam_kernel(f4* __restrict__ x, f4* __restrict__ m,
                                                   f4* __restrict__ v, const f4* __restrict__ g,
                                                   int64_t n4, UpdateRule rule) {
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
    f4 p = x[i], a = m[i], b = v[i];
    const f4 d = g[i];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float ae = a[e], be = b[e];
      p[e] = step_one<DYNB_OPT_ADAM>(rule, p[e], d[e], ae, be);
      a[e] = ae;
      b[e] = be;
    }
    x[i] = p;
    m[i] = a;
    v[i] = b;
  }
}

inline int ok(const char* what) {
  return hipGetLastError() == hipSuccess ? DYNB_OK : fail(DYNB_ERR_HIP, "%s: launch failed", what);
}

// algorithmic bytes per parameter of one step: parameter read + write, each state read + write,
// and the gradient (one read, or K reads when aggregating on the fly)
double bytes_per_param(const UpdateRule& rule, const GradSource& src) {
  const int states = rule.kind == DYNB_OPT_ADAM ? 2 : rule.kind == DYNB_OPT_MOMENTUM ? 1 : 0;
  return 8.0 + 8.0 * states + 4.0 * (src.lam.K > 0 ? src.lam.K : 1);
}
double flops_per_param(const UpdateRule& rule, const GradSource& src) {
  const double step = rule.kind == DYNB_OPT_ADAM ? 14.0 : rule.kind == DYNB_OPT_MOMENTUM ? 4.0 : 2.0;
  return step + (src.lam.K > 0 ? 2.0 * src.lam.K : 0.0);
}

// (wider tiles when K gradient streams are read: 512-byte runs per row and stream)
constexpr int cast_tile_columns(bool agg) { return agg ? 128 : 64; }

template <typename T, int KIND, bool AGG>
void launch_update_cast_t(float* params, const CastMats& mats, const Ranges& small, int range_blocks,
                          const GradSource& src, const UpdateRule& rule, float* s1, float* s2,
                          hipStream_t st) {
  constexpr int TC = cast_tile_columns(AGG);
  const dim3 grid((unsigned)(mats.first_block[mats.n] + range_blocks));
  hipLaunchKernelGGL((update_cast_kernel<T, KIND, AGG, TC>), grid, dim3(256), 0, st, params, mats, small,
                     range_blocks, src, rule, s1, s2);
}

template <typename T, int KIND>
void launch_update_cast_k(float* params, const CastMats& mats, const Ranges& small, int range_blocks,
                          const GradSource& src, const UpdateRule& rule, float* s1, float* s2,
                          hipStream_t st) {
  if (src.lam.K > 0)
    launch_update_cast_t<T, KIND, true>(params, mats, small, range_blocks, src, rule, s1, s2, st);
  else
    launch_update_cast_t<T, KIND, false>(params, mats, small, range_blocks, src, rule, s1, s2, st);
}

template <typename T>
void launch_update_cast_d(float* params, const CastMats& mats, const Ranges& small, int range_blocks,
                          const GradSource& src, const UpdateRule& rule, float* s1, float* s2,
                          hipStream_t st) {
  switch (rule.kind) {
    case DYNB_OPT_SGD:
      launch_update_cast_k<T, DYNB_OPT_SGD>(params, mats, small, range_blocks, src, rule, s1, s2, st);
      break;
    case DYNB_OPT_MOMENTUM:
      launch_update_cast_k<T, DYNB_OPT_MOMENTUM>(params, mats, small, range_blocks, src, rule, s1, s2, st);
      break;
    default:
      launch_update_cast_k<T, DYNB_OPT_ADAM>(params, mats, small, range_blocks, src, rule, s1, s2, st);
  }
}

template <int KIND>
void launch_update_range_k(float* params, int64_t off, const GradSource& src, const UpdateRule& rule,
                           float* s1, float* s2, int64_t n, unsigned bx, hipStream_t st) {
  if (src.lam.K > 0)
    hipLaunchKernelGGL((update_range_kernel<KIND, true>), dim3(bx), dim3(256), 0, st, params, off, src,
                       rule, s1, s2, n);
  else
    hipLaunchKernelGGL((update_range_kernel<KIND, false>), dim3(bx), dim3(256), 0, st, params, off, src,
                       rule, s1, s2, n);
}

}  // namespace

int launch_update_cast(int dtype, float* params, CastMats& mats, const Ranges& small,
                       const GradSource& src, const UpdateRule& rule, float* s1, float* s2,
                       void* stream) {
  if (mats.n < 0 || mats.n > MAX_CAST_MATS || small.n < 0 || small.n > MAX_RANGES)
    return fail(DYNB_ERR_BADARG, "update_cast: too many tensors for one launch");
  const int es = dtype == DYNB_BF16 ? 2 : 4;
  const int TC = cast_tile_columns(src.lam.K > 0);
  double cast_n = 0.0, small_n = 0.0;
  int64_t blocks = 0, longest = 0;
  for (int i = 0; i < mats.n; ++i) {
    if (mats.R[i] <= 0 || mats.C[i] <= 0) return fail(DYNB_ERR_BADARG, "update_cast: empty matrix");
    mats.first_block[i] = (int)blocks;
    blocks += (int64_t)((mats.C[i] + TC - 1) / TC) * ((mats.R[i] + 63) / 64);
    cast_n += (double)mats.R[i] * mats.C[i];
  }
  for (int i = 0; i < small.n; ++i) {
    longest = small.len[i] > longest ? small.len[i] : longest;
    small_n += (double)small.len[i];
  }
  int64_t range_blocks = (longest + 255) / 256;
  if (range_blocks > 256) range_blocks = 256;
  if (blocks + range_blocks >= ((int64_t)1 << 31))
    return fail(DYNB_ERR_UNSUPPORTED, "update_cast: too many tiles for one launch");
  if (blocks + range_blocks == 0) return DYNB_OK;
  for (int i = mats.n; i <= MAX_CAST_MATS; ++i) mats.first_block[i] = (int)blocks;
  Timed t(KC_UPDATE, stream, flops_per_param(rule, src) * (cast_n + small_n),
          (bytes_per_param(rule, src) + 2 * es) * cast_n + bytes_per_param(rule, src) * small_n);
  if (dtype == DYNB_BF16)
    launch_update_cast_d<bf16>(params, mats, small, (int)range_blocks, src, rule, s1, s2, (hipStream_t)stream);
  else
    launch_update_cast_d<float>(params, mats, small, (int)range_blocks, src, rule, s1, s2, (hipStream_t)stream);
  return ok("update_cast");
}

int launch_update_range(float* params, int64_t off, const GradSource& src, const UpdateRule& rule,
                        float* s1, float* s2, int64_t n, void* stream) {
  if (n <= 0) return DYNB_OK;
  Timed t(KC_UPDATE, stream, flops_per_param(rule, src) * n, bytes_per_param(rule, src) * n);
  int64_t bx = (n + 255) / 256;
  if (bx > 2048) bx = 2048;
  switch (rule.kind) {
    case DYNB_OPT_SGD:
      launch_update_range_k<DYNB_OPT_SGD>(params, off, src, rule, s1, s2, n, (unsigned)bx, (hipStream_t)stream);
      break;
    case DYNB_OPT_MOMENTUM:
      launch_update_range_k<DYNB_OPT_MOMENTUM>(params, off, src, rule, s1, s2, n, (unsigned)bx, (hipStream_t)stream);
      break;
    default:
      launch_update_range_k<DYNB_OPT_ADAM>(params, off, src, rule, s1, s2, n, (unsigned)bx, (hipStream_t)stream);
  }
  return ok("update_range");
}

void set_adam(UpdateRule& r, double beta1, double beta2, float eps, int64_t t) {
  r.beta1 = (float)beta1;
  r.beta2 = (float)beta2;
  r.omb1 = (float)(1.0 - beta1);
  r.omb2 = (float)(1.0 - beta2);
  r.eps = eps;
  r.inv_c1 = (float)(1.0 / (1.0 - std::pow(beta1, (double)t)));
  r.inv_c2 = (float)(1.0 / (1.0 - std::pow(beta2, (double)t)));
}

namespace {
template <int KIND>
void launch_update_ranges_k(float* params, const Ranges& r, const GradSource& src, const UpdateRule& rule,
                            float* s1, float* s2, dim3 grid, hipStream_t st) {
  if (src.lam.K > 0)
    hipLaunchKernelGGL((update_ranges_kernel<KIND, true>), grid, dim3(256), 0, st, params, r, src, rule, s1, s2);
  else
    hipLaunchKernelGGL((update_ranges_kernel<KIND, false>), grid, dim3(256), 0, st, params, r, src, rule, s1, s2);
}
}  // namespace

int launch_update_ranges(float* params, const Ranges& r, const GradSource& src, const UpdateRule& rule,
                         float* s1, float* s2, void* stream) {
  int64_t longest = 0, total = 0;
  for (int i = 0; i < r.n; ++i) {
    longest = r.len[i] > longest ? r.len[i] : longest;
    total += r.len[i];
  }
  if (r.n <= 0 || longest <= 0) return DYNB_OK;
  Timed t(KC_UPDATE, stream, flops_per_param(rule, src) * total, bytes_per_param(rule, src) * total);
  int64_t bx = (longest + 255) / 256;
  if (bx > 1024) bx = 1024;
  const dim3 grid((unsigned)bx, r.n);
  switch (rule.kind) {
    case DYNB_OPT_SGD:
      launch_update_ranges_k<DYNB_OPT_SGD>(params, r, src, rule, s1, s2, grid, (hipStream_t)stream);
      break;
    case DYNB_OPT_MOMENTUM:
      launch_update_ranges_k<DYNB_OPT_MOMENTUM>(params, r, src, rule, s1, s2, grid, (hipStream_t)stream);
      break;
    default:
      launch_update_ranges_k<DYNB_OPT_ADAM>(params, r, src, rule, s1, s2, grid, (hipStream_t)stream);
  }
  return ok("update_ranges");
}

int launch_adam(float* params, float* m, float* v, const float* g, int64_t n,
                const UpdateRule& rule, void* stream) {
  const int64_t n4 = n / 4;
  if (n4 == 0) return DYNB_OK;
  Timed t(KC_UPDATE, stream, 14.0 * n, 28.0 * n);
  int64_t bx = (n4 + 255) / 256;
  if (bx > 256 * 16) bx = 256 * 16;
  hipLaunchKernelGGL(adam_kernel, dim3((unsigned)bx), dim3(256), 0, (hipStream_t)stream, (f4*)params,
                     (f4*)m, (f4*)v, (const f4*)g, n4, rule);
  return ok("adam");
}

}  // namespace dynb

using namespace dynb;

extern "C" int dynb_adam_update(float* params, float* m, float* v, const float* g, int64_t n,
                                float lr, double beta1, double beta2, float eps, int64_t step,
                                void* stream) {
  if (!params || !m || !v || !g) return fail(DYNB_ERR_BADARG, "adam: null pointer");
  if (n < 0 || (n & 3)) return fail(DYNB_ERR_BADARG, "adam: n must be a non-negative multiple of 4");
  if (((uintptr_t)params | (uintptr_t)m | (uintptr_t)v | (uintptr_t)g) & 15)
    return fail(DYNB_ERR_BADARG, "adam: pointers must be 16-byte aligned");
  if (step < 1) return fail(DYNB_ERR_BADARG, "adam: step numbers start at 1");
  if (!(beta1 >= 0.0 && beta1 < 1.0 && beta2 >= 0.0 && beta2 < 1.0))
    return fail(DYNB_ERR_BADARG, "adam: betas must lie in [0, 1)");
  UpdateRule r{};
  r.kind = DYNB_OPT_ADAM;
  r.lr = lr;
  set_adam(r, beta1, beta2, eps, step);
  return launch_adam(params, m, v, g, n, r, stream);
}
