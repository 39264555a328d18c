// Batch normalisation over each worker's own rows and residual additions (bf16 storage).
// A "row" is a sample or a pixel; worker k owns rows [off_k, off_{k+1}).  The statistics of a
// worker never see another worker's rows, so every reduction here runs per (worker, channel).
// The rows of a worker are cut into chunks of CHUNK_ROWS; one workgroup takes one chunk and 64
// channels (a lane: 8 channels of a row = one 16-byte access, 8 lanes = the 128 bytes of a row,
// 32 rows per pass), writes the chunk's partial result, and a second small kernel merges the
// chunks of each worker in a fixed order.  All sums are fp32 and deterministic.
#include <hip/hip_runtime.h>

#include "device_rows.h"
#include "dynb_internal.h"

namespace dynb {
namespace {

constexpr int CHUNK_ROWS = BN_CHUNK_ROWS;
constexpr int PASSES = CHUNK_ROWS / 32;

// first[k] = index of worker k's first chunk; first[K] = number of chunks
struct Chunks {
  int first[DYNB_MAX_WORKERS + 1];
};

// worker, first row and row count of a chunk (chunk < first[K], so the scan ends)
__device__ inline void chunk_span(const Segs& s, const Chunks& ch, int chunk, int& k, int& r0, int& n) {
  k = 0;
  while (k + 1 < s.K && chunk >= ch.first[k + 1]) ++k;
  r0 = s.off[k] + (chunk - ch.first[k]) * CHUNK_ROWS;
  n = min(CHUNK_ROWS, s.off[k + 1] - r0);
}

// Mean and sum of centred squares of one chunk (its values stay in registers between the two).
__global__ __launch_bounds__(256) void bn_chunk_stats_kernel(const bf16* __restrict__ x, int64_t ld,
                                                             int C, float* __restrict__ pmean,
                                                             float* __restrict__ pm2, Segs s, Chunks ch) {
  __shared__ float red[4][64];
  const int cg = threadIdx.x & 7, rl = threadIdx.x >> 3;
  const int chunk = blockIdx.x, c0 = blockIdx.y * 64 + cg * 8;
  int k, r0, n;
  chunk_span(s, ch, chunk, k, r0, n);
  const bf16* base = x + (int64_t)r0 * ld + c0;
  float v[PASSES][8], acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) acc[j] = 0.f;
#pragma unroll
  for (int i = 0; i < PASSES; ++i) {
    const int r = rl + 32 * i;
    const uint4 q = r < n ? load8(base + (int64_t)r * ld) : make_uint4(0, 0, 0, 0);
    unpack8(q, v[i]);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] += v[i][j];
  }
  sum_over_rows(acc, red);
  float mu[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) { mu[j] = acc[j] / (float)n; acc[j] = 0.f; }
#pragma unroll
  for (int i = 0; i < PASSES; ++i) {
    if (rl + 32 * i < n) {
#pragma unroll
      for (int j = 0; j < 8; ++j) { const float d = v[i][j] - mu[j]; acc[j] += d * d; }
    }
  }
  sum_over_rows(acc, red);
  if (rl == 0) {
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (c0 + j < C) {
        pmean[(int64_t)chunk * C + c0 + j] = mu[j];
        pm2[(int64_t)chunk * C + c0 + j] = acc[j];
      }
  }
}

// Sum over the chunks of one worker, for 64 channels at a time: 1024 threads = 64 channels x 16
// chunk-lanes; lane q adds the terms of chunks q, q+16, ... (four independent partial sums, so
// that the loads overlap), the 16 lanes are then added in ascending order.  term(j) = value of
// chunk j for this thread's channel.  Every thread of the channel gets the total.
template <typename F>
__device__ inline float sum_over_chunks(int nc, int q, int cl, float (*red)[64], F term) {
  float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
  int j = q;
  for (; j + 48 < nc; j += 64) {
    a0 += term(j); a1 += term(j + 16); a2 += term(j + 32); a3 += term(j + 48);
  }
  for (; j < nc; j += 16) a0 += term(j);
  __syncthreads();
  red[q][cl] = (a0 + a1) + (a2 + a3);
  __syncthreads();
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) t += red[i][cl];
  return t;
}

// mean[k][c], rstd[k][c] from the chunk moments of worker k: the mean is the weighted sum of
// the chunk means, the sum of squares follows from the parallel-axis relation
//   M2 = sum_j (M2_j + n_j (mean_j - mean)^2)
// -- two plain sums in a fixed order.
__global__ __launch_bounds__(1024) void bn_merge_stats_kernel(const float* __restrict__ pmean,
                                                              const float* __restrict__ pm2, int C,
                                                              float eps, float* __restrict__ mean,
                                                              float* __restrict__ rstd, Segs s, Chunks ch) {
  __shared__ float red[16][64];
  const int cl = threadIdx.x & 63, q = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + cl, k = blockIdx.y;
  const int rows = s.off[k + 1] - s.off[k];
  if (rows <= 0) return;                      // (uniform over the workgroup)
  const int first = ch.first[k], nc = ch.first[k + 1] - first;
  const int cc = c < C ? c : C - 1;           // lanes past the last channel repeat it, unused
  const float n = (float)rows;
  auto rows_of = [&](int j) { return (float)min(CHUNK_ROWS, rows - j * CHUNK_ROWS); };
  const float mu = sum_over_chunks(nc, q, cl, red, [&](int j) {
                     return rows_of(j) * pmean[(int64_t)(first + j) * C + cc];
                   }) / n;
  const float m2 = sum_over_chunks(nc, q, cl, red, [&](int j) {
    const float d = pmean[(int64_t)(first + j) * C + cc] - mu;
    return pm2[(int64_t)(first + j) * C + cc] + rows_of(j) * d * d;
  });
  if (q == 0 && c < C) {
    mean[(int64_t)k * C + c] = mu;
    rstd[(int64_t)k * C + c] = 1.f / sqrtf(m2 / n + eps);
  }
}

// y = relu?(gamma * ((x - mean_k) * rstd_k) + beta); padding channels are written as zero.
// With `skip`, the residual addition behind the normalisation is applied in the same pass:
// y = relu_sum?(bf16(normalised) + skip) -- rounded as if the normalised tensor had been stored.
__global__ __launch_bounds__(256) void bn_apply_kernel(const bf16* __restrict__ x, int64_t ldx, int C,
                                                       const float* __restrict__ gamma,
                                                       const float* __restrict__ beta,
                                                       const float* __restrict__ mean,
                                                       const float* __restrict__ rstd, int relu,
                                                       const bf16* __restrict__ skip, int64_t lds_,
                                                       int relu_sum, bf16* __restrict__ y, int64_t ldy,
                                                       Segs s, Chunks ch) {
  const int cg = threadIdx.x & 7, rl = threadIdx.x >> 3;
  const int chunk = blockIdx.x, c0 = blockIdx.y * 64 + cg * 8;
  int k, r0, n;
  chunk_span(s, ch, chunk, k, r0, n);
  float mu[8], rs[8], ga[8], be[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    // (clamped index, then a select: all loads are issued at once, no branch per channel)
    const bool live = c0 + j < C;
    const int cj = live ? c0 + j : C - 1;
    const float m_ = mean[(int64_t)k * C + cj], r_ = rstd[(int64_t)k * C + cj];
    const float g_ = gamma[cj], b_ = beta[cj];
    mu[j] = live ? m_ : 0.f;
    rs[j] = live ? r_ : 0.f;
    ga[j] = live ? g_ : 0.f;
    be[j] = live ? b_ : 0.f;
  }
  const bf16* xb = x + (int64_t)r0 * ldx + c0;
  bf16* yb = y + (int64_t)r0 * ldy + c0;
#pragma unroll
  for (int i = 0; i < PASSES; ++i) {
    const int r = rl + 32 * i;
    if (r < n) {
      float v[8];
      unpack8(load8(xb + (int64_t)r * ldx), v);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        float t = ga[j] * ((v[j] - mu[j]) * rs[j]) + be[j];
        if (relu) t = fmaxf(t, 0.f);
        v[j] = c0 + j < C ? t : 0.f;
      }
      if (skip) {
        float u[8], w[8];
        unpack8(pack8(v), u);                    // the normalised values as they would be stored
        unpack8(load8(skip + (int64_t)(r0 + r) * lds_ + c0), w);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          v[j] = u[j] + w[j];
          if (relu_sum) v[j] = fmaxf(v[j], 0.f);
        }
      }
      store8(yb + (int64_t)r * ldy, pack8(v));
    }
  }
}

// Chunk sums of dy and of dy * xhat (dy already carries this layer's ReLU mask).
__global__ __launch_bounds__(256) void bn_chunk_param_grad_kernel(
    const bf16* __restrict__ dy, int64_t ldd, const bf16* __restrict__ x, int64_t ldx, int C,
    const float* __restrict__ mean, const float* __restrict__ rstd, float* __restrict__ pdg,
    float* __restrict__ pdb, Segs s, Chunks ch) {
  __shared__ float red[4][64];
  const int cg = threadIdx.x & 7, rl = threadIdx.x >> 3;
  const int chunk = blockIdx.x, c0 = blockIdx.y * 64 + cg * 8;
  int k, r0, n;
  chunk_span(s, ch, chunk, k, r0, n);
  float mu[8], rs[8], ag[8], ab[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const bool live = c0 + j < C;
    const int cj = live ? c0 + j : C - 1;
    const float m_ = mean[(int64_t)k * C + cj], r_ = rstd[(int64_t)k * C + cj];
    mu[j] = live ? m_ : 0.f;
    rs[j] = live ? r_ : 0.f;
    ag[j] = 0.f; ab[j] = 0.f;
  }
  const bf16* xb = x + (int64_t)r0 * ldx + c0;
  const bf16* db = dy + (int64_t)r0 * ldd + c0;
#pragma unroll
  for (int i = 0; i < PASSES; ++i) {
    const int r = rl + 32 * i;
    if (r < n) {
      float v[8], d[8];
      unpack8(load8(xb + (int64_t)r * ldx), v);
      unpack8(load8(db + (int64_t)r * ldd), d);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        ab[j] += d[j];
        ag[j] += d[j] * ((v[j] - mu[j]) * rs[j]);
      }
    }
  }
  sum_over_rows(ag, red);
  sum_over_rows(ab, red);
  if (rl == 0) {
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (c0 + j < C) {
        pdg[(int64_t)chunk * C + c0 + j] = ag[j];
        pdb[(int64_t)chunk * C + c0 + j] = ab[j];
      }
  }
}

// dgamma[k][c], dbeta[k][c] = the chunk sums of worker k added in a fixed order, written into
// worker k's gradient vector; a worker without rows gets zeros.
__global__ __launch_bounds__(1024) void bn_merge_param_grad_kernel(const float* __restrict__ pdg,
                                                                   const float* __restrict__ pdb, int C,
                                                                   float* __restrict__ dgamma,
                                                                   float* __restrict__ dbeta,
                                                                   int64_t group_stride, Chunks ch) {
  __shared__ float red[16][64];
  const int cl = threadIdx.x & 63, q = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + cl, k = blockIdx.y;
  const int first = ch.first[k], nc = ch.first[k + 1] - first;
  const int cc = c < C ? c : C - 1;
  const float g = sum_over_chunks(nc, q, cl, red, [&](int j) { return pdg[(int64_t)(first + j) * C + cc]; });
  const float b = sum_over_chunks(nc, q, cl, red, [&](int j) { return pdb[(int64_t)(first + j) * C + cc]; });
  if (q == 0 && c < C) {
    dgamma[(int64_t)k * group_stride + c] = g;
    dbeta[(int64_t)k * group_stride + c] = b;
  }
}

// dx = gamma * rstd * (dy - dbeta/n - xhat * dgamma/n), masked by the producer's ReLU (x > 0);
// padding channels are written as zero
__global__ __launch_bounds__(256) void bn_input_grad_kernel(
    const bf16* __restrict__ dy, int64_t ldd, const bf16* __restrict__ x, int64_t ldx, int C,
    const float* __restrict__ gamma, const float* __restrict__ mean, const float* __restrict__ rstd,
    const float* __restrict__ dgamma, const float* __restrict__ dbeta, int64_t group_stride,
    int relu_below, bf16* __restrict__ dx, int64_t ldo, Segs s, Chunks ch) {
  const int cg = threadIdx.x & 7, rl = threadIdx.x >> 3;
  const int chunk = blockIdx.x, c0 = blockIdx.y * 64 + cg * 8;
  int k, r0, n;
  chunk_span(s, ch, chunk, k, r0, n);
  const float rows = (float)(s.off[k + 1] - s.off[k]);
  float mu[8], rs[8], gr[8], mg[8], mb[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const bool live = c0 + j < C;
    const int cj = live ? c0 + j : C - 1;
    const float m_ = mean[(int64_t)k * C + cj], r_ = rstd[(int64_t)k * C + cj], g_ = gamma[cj];
    const float dg_ = dgamma[(int64_t)k * group_stride + cj], db_ = dbeta[(int64_t)k * group_stride + cj];
    mu[j] = live ? m_ : 0.f;
    rs[j] = live ? r_ : 0.f;
    gr[j] = live ? g_ * r_ : 0.f;
    mg[j] = live ? dg_ / rows : 0.f;
    mb[j] = live ? db_ / rows : 0.f;
  }
  const bf16* xb = x + (int64_t)r0 * ldx + c0;
  const bf16* db = dy + (int64_t)r0 * ldd + c0;
  bf16* ob = dx + (int64_t)r0 * ldo + c0;
#pragma unroll
  for (int i = 0; i < PASSES; ++i) {
    const int r = rl + 32 * i;
    if (r < n) {
      float v[8], d[8];
      unpack8(load8(xb + (int64_t)r * ldx), v);
      unpack8(load8(db + (int64_t)r * ldd), d);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        float t = gr[j] * (d[j] - mb[j] - ((v[j] - mu[j]) * rs[j]) * mg[j]);
        if (relu_below && !(v[j] > 0.f)) t = 0.f;
        d[j] = c0 + j < C ? t : 0.f;
      }
      store8(ob + (int64_t)r * ldo, pack8(d));
    }
  }
}

// Element-wise kernels: one lane takes 8 channels of a row; `gpr` = 16-byte granules per row
// (the padded width / 8; padding channels hold zeros on both sides).

// out = relu?(a + b)
__global__ __launch_bounds__(256) void add_forward_kernel(const bf16* __restrict__ a, int64_t lda,
                                                          const bf16* __restrict__ b, int64_t ldb,
                                                          int gpr, int64_t total, int relu,
                                                          bf16* __restrict__ out, int64_t ldo) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int64_t row = i / gpr;
  const int c0 = (int)(i - row * gpr) * 8;
  float u[8], v[8];
  unpack8(load8(a + row * lda + c0), u);
  unpack8(load8(b + row * ldb + c0), v);
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    u[j] += v[j];
    if (relu) u[j] = fmaxf(u[j], 0.f);
  }
  store8(out + row * ldo + c0, pack8(u));
}

// dst = (accumulate ? dst : 0) + src, masked by act > 0 when `relu` (act = the stored output of
// the layer whose gradient dst is)
__global__ __launch_bounds__(256) void grad_route_kernel(const bf16* __restrict__ src, int64_t lds_,
                                                         const bf16* __restrict__ act, int64_t lda,
                                                         int gpr, int64_t total, int relu,
                                                         int accumulate, bf16* __restrict__ dst,
                                                         int64_t ldd) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int64_t row = i / gpr;
  const int c0 = (int)(i - row * gpr) * 8;
  float v[8];
  unpack8(load8(src + row * lds_ + c0), v);
  if (relu) {
    float a[8];
    unpack8(load8(act + row * lda + c0), a);
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (!(a[j] > 0.f)) v[j] = 0.f;
  }
  if (accumulate) {
    float d[8];
    unpack8(load8(dst + row * ldd + c0), d);
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] += d[j];
  }
  store8(dst + row * ldd + c0, pack8(v));
}

inline int ok(const char* what) {
  return hipGetLastError() == hipSuccess ? DYNB_OK : fail(DYNB_ERR_HIP, "%s: launch failed", what);
}

Chunks make_chunks(const Segs& s) {
  Chunks ch;
  ch.first[0] = 0;
  for (int k = 0; k < s.K; ++k)
    ch.first[k + 1] = ch.first[k] + (s.off[k + 1] - s.off[k] + CHUNK_ROWS - 1) / CHUNK_ROWS;
  for (int k = s.K + 1; k <= DYNB_MAX_WORKERS; ++k) ch.first[k] = ch.first[s.K];
  return ch;
}

}  // namespace

int launch_bn_forward(const void* x, int64_t ldx, int C, const float* gamma, const float* beta,
                      float eps, int relu, float* mean, float* rstd, float* scratch,
                      const void* skip, int64_t lds_, int relu_sum, void* y, int64_t ldy,
                      const Segs& s, void* stream) {
  const int rows = s.off[s.K];
  if (rows == 0 || C == 0) return DYNB_OK;
  const Chunks ch = make_chunks(s);
  const int nch = ch.first[s.K], cb = (C + 63) / 64;
  float* pmean = scratch;
  float* pm2 = scratch + (int64_t)nch * C;
  // algorithmic bytes: x read and y written once (+ the skip tensor); the statistics pass reads x again
  Timed t(KC_NORM, stream, 0, (double)rows * C * (skip ? 6 : 4));
  hipLaunchKernelGGL(bn_chunk_stats_kernel, dim3(nch, cb), dim3(256), 0, (hipStream_t)stream,
                     (const bf16*)x, ldx, C, pmean, pm2, s, ch);
  hipLaunchKernelGGL(bn_merge_stats_kernel, dim3(cb, s.K), dim3(1024), 0, (hipStream_t)stream, pmean,
                     pm2, C, eps, mean, rstd, s, ch);
  hipLaunchKernelGGL(bn_apply_kernel, dim3(nch, (unsigned)(ldy / 64)), dim3(256), 0,
                     (hipStream_t)stream, (const bf16*)x, ldx, C, gamma, beta, mean, rstd, relu,
                     (const bf16*)skip, lds_, relu_sum, (bf16*)y, ldy, s, ch);
  return ok("bn_forward");
}

int launch_bn_backward(const void* dy, int64_t ldd, const void* x, int64_t ldx, int C,
                       const float* gamma, const float* mean, const float* rstd, float* scratch,
                       float* dgamma, float* dbeta, int64_t group_stride, int need_dx,
                       int relu_below, void* dx, int64_t ldo, const Segs& s, void* stream) {
  const int rows = s.off[s.K];
  if (C == 0) return DYNB_OK;
  const Chunks ch = make_chunks(s);
  const int nch = ch.first[s.K], cb = (C + 63) / 64;
  float* pdg = scratch;
  float* pdb = scratch + (int64_t)nch * C;
  // algorithmic bytes: dy and x read once, dx written once (the kernels read dy and x twice)
  Timed t(KC_NORM, stream, 0, (double)rows * C * (need_dx ? 6 : 4));
  if (nch > 0)
    hipLaunchKernelGGL(bn_chunk_param_grad_kernel, dim3(nch, cb), dim3(256), 0, (hipStream_t)stream,
                       (const bf16*)dy, ldd, (const bf16*)x, ldx, C, mean, rstd, pdg, pdb, s, ch);
  hipLaunchKernelGGL(bn_merge_param_grad_kernel, dim3(cb, s.K), dim3(1024), 0, (hipStream_t)stream, pdg,
                     pdb, C, dgamma, dbeta, group_stride, ch);
  if (need_dx && nch > 0)
    hipLaunchKernelGGL(bn_input_grad_kernel, dim3(nch, (unsigned)(ldo / 64)), dim3(256), 0,
                       (hipStream_t)stream, (const bf16*)dy, ldd, (const bf16*)x, ldx, C, gamma, mean,
                       rstd, dgamma, dbeta, group_stride, relu_below, (bf16*)dx, ldo, s, ch);
  return ok("bn_backward");
}

int64_t row_scratch_floats(int64_t max_rows, int max_workers, int C) {
  return 2 * ((max_rows + CHUNK_ROWS - 1) / CHUNK_ROWS + max_workers) * (int64_t)C;
}

int launch_add_forward(const void* a, int64_t lda, const void* b, int64_t ldb, int64_t width,
                       int64_t rows, int relu, void* out, int64_t ldo, void* stream) {
  if (rows == 0 || width == 0) return DYNB_OK;
  const int gpr = (int)(width / 8);
  const int64_t total = rows * gpr;
  Timed t(KC_NORM, stream, 0, (double)rows * width * 6);
  hipLaunchKernelGGL(add_forward_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                     (hipStream_t)stream, (const bf16*)a, lda, (const bf16*)b, ldb, gpr, total, relu,
                     (bf16*)out, ldo);
  return ok("add_forward");
}

int launch_grad_route(const void* src, int64_t lds_, const void* act, int64_t lda, int64_t width,
                      int64_t rows, int relu, int accumulate, void* dst, int64_t ldd, void* stream) {
  if (rows == 0 || width == 0) return DYNB_OK;
  const int gpr = (int)(width / 8);
  const int64_t total = rows * gpr;
  Timed t(KC_NORM, stream, 0, (double)rows * width * (2 + 2 + (relu ? 2 : 0) + (accumulate ? 2 : 0)));
  hipLaunchKernelGGL(grad_route_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                     (hipStream_t)stream, (const bf16*)src, lds_, (const bf16*)act, lda, gpr, total,
                     relu, accumulate, (bf16*)dst, ldd);
  return ok("grad_route");
}

}  // namespace dynb
