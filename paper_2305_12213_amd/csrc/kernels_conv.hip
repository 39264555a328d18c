// Kernels around the implicit-GEMM convolutions (NHWC, 3x3, zero padding 1; bf16 storage):
// global average pooling forward/backward and the two 16-bit weight layouts of a convolution.
#include <hip/hip_runtime.h>

#include "device_rows.h"
#include "dynb_internal.h"

namespace dynb {
namespace {

// pooled[n][c] = mean over the HW pixels of act[(n, pixel)][c]   (fp32 sum in a fixed order,
// bf16 store).  One workgroup per (sample, 64 channels); padding channels are written as zero.
__global__ __launch_bounds__(256) void gap_forward_kernel(const bf16* __restrict__ act, int64_t lda,
                                                          int HW, int C, bf16* __restrict__ pooled,
                                                          int64_t ldp) {
  __shared__ float red[4][64];
  const int cg = threadIdx.x & 7, rl = threadIdx.x >> 3;
  const int n = blockIdx.x, c0 = blockIdx.y * 64 + cg * 8;
  const bf16* base = act + (int64_t)n * HW * lda + c0;
  float acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) acc[j] = 0.f;
  for (int px = rl; px < HW; px += 32) {
    float v[8];
    unpack8(load8(base + (int64_t)px * lda), v);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] += v[j];
  }
  sum_over_rows(acc, red);
  if (rl == 0) {
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = c0 + j < C ? acc[j] / (float)HW : 0.f;
    store8(pooled + (int64_t)n * ldp + c0, pack8(acc));
  }
}

// d act[(n, pixel)][c] = d pooled[n][c] / HW, masked by act > 0 when the pooled layer's producer
// applied a ReLU.  One lane per 8 channels of a row; `gpr` = 16-byte granules per row.
__global__ __launch_bounds__(256) void gap_backward_kernel(const bf16* __restrict__ dpooled,
                                                           int64_t ldp, const bf16* __restrict__ act,
                                                           int64_t lda, int HW, int gpr, int64_t total,
                                                           int relu, bf16* __restrict__ dact,
                                                           int64_t ldd) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int64_t row = i / gpr;   // (n, pixel)
  const int c0 = (int)(i - row * gpr) * 8;
  float v[8];
  unpack8(load8(dpooled + (row / HW) * ldp + c0), v);
#pragma unroll
  for (int j = 0; j < 8; ++j) v[j] = v[j] / (float)HW;
  if (relu) {
    float a[8];
    unpack8(load8(act + row * lda + c0), a);
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (!(a[j] > 0.f)) v[j] = 0.f;
  }
  store8(dact + row * ldd + c0, pack8(v));
}

// W fp32 [3][3][Cin][Cout] ->
//   Wf [Cout][kf] : Wf[co][(kh*3+kw)*cin_p + ci] = W[kh][kw][ci][co]   (forward B operand)
//   Wd [Cin][kd]  : Wd[ci][(kh*3+kw)*cout_p + co] = W[kh][kw][ci][co]  (input-gradient B operand)
// Positions that correspond to padded channels or padded reduction length are written as zero.
__global__ __launch_bounds__(256) void conv_weight_cast_kernel(const float* __restrict__ W, int Cin,
                                                               int Cout, int cin_p, int cout_p,
                                                               bf16* __restrict__ Wf, int kf,
                                                               bf16* __restrict__ Wd, int kd) {
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t nf = (int64_t)Cout * kf, nd = (int64_t)Cin * kd;
  if (t < nf) {
    const int co = (int)(t / kf), k = (int)(t - (int64_t)co * kf);
    const int tap = k / cin_p, ci = k - tap * cin_p;
    float v = 0.f;
    if (tap < 9 && ci < Cin) v = W[((int64_t)tap * Cin + ci) * Cout + co];
    Wf[t] = (bf16)v;
  } else if (t < nf + nd) {
    const int64_t u = t - nf;
    const int ci = (int)(u / kd), k = (int)(u - (int64_t)ci * kd);
    const int tap = k / cout_p, co = k - tap * cout_p;
    float v = 0.f;
    if (tap < 9 && co < Cout) v = W[((int64_t)tap * Cin + ci) * Cout + co];
    Wd[u] = (bf16)v;
  }
}

inline int ok(const char* what) {
  return hipGetLastError() == hipSuccess ? DYNB_OK : fail(DYNB_ERR_HIP, "%s: launch failed", what);
}

}  // namespace

int launch_gap_forward(const void* act, int64_t lda, int HW, int C, int samples, void* pooled,
                       int64_t ldp, void* stream) {
  if (samples == 0) return DYNB_OK;
  if (lda % 64 || ldp % 64 || lda < ldp) return fail(DYNB_ERR_BADARG, "gap_forward: bad pitches");
  Timed t(KC_CONV_AUX, stream, 0, (double)samples * HW * C * 2);
  dim3 grid(samples, (unsigned)(ldp / 64));
  hipLaunchKernelGGL(gap_forward_kernel, grid, dim3(256), 0, (hipStream_t)stream, (const bf16*)act,
                     lda, HW, C, (bf16*)pooled, ldp);
  return ok("gap_forward");
}

int launch_gap_backward(const void* dpooled, int64_t ldp, const void* act, int64_t lda, int HW,
                        int C, int samples, int relu, void* dact, int64_t ldd, void* stream) {
  if (samples == 0) return DYNB_OK;
  if (lda % 64 || ldp % 64 || ldd % 64 || ldp < ldd || lda < ldd)
    return fail(DYNB_ERR_BADARG, "gap_backward: bad pitches");
  const int gpr = (int)(ldd / 8);
  const int64_t total = (int64_t)samples * HW * gpr;
  Timed t(KC_CONV_AUX, stream, 0, (double)samples * HW * C * 4);
  hipLaunchKernelGGL(gap_backward_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                     (hipStream_t)stream, (const bf16*)dpooled, ldp, (const bf16*)act, lda, HW, gpr,
                     total, relu, (bf16*)dact, ldd);
  return ok("gap_backward");
}

int launch_conv_weight_cast(const float* W, int Cin, int Cout, int cin_p, int cout_p, void* Wf,
                            int kf, void* Wd, int kd, void* stream) {
  const int64_t total = (int64_t)Cout * kf + (int64_t)Cin * kd;
  Timed t(KC_WEIGHT_CAST, stream, 0, 9.0 * Cin * Cout * 4 + total * 2);
  hipLaunchKernelGGL(conv_weight_cast_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                     (hipStream_t)stream, W, Cin, Cout, cin_p, cout_p, (bf16*)Wf, kf, (bf16*)Wd, kd);
  return ok("conv_weight_cast");
}

}  // namespace dynb
