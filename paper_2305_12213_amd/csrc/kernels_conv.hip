// Kernels around the implicit-GEMM convolutions (NHWC, 3x3, zero padding 1; bf16 storage):
// the transposed patch matrix that feeds the per-worker weight-gradient GEMM, global average
// pooling forward/backward, and the two 16-bit weight layouts of a convolution.
#include <hip/hip_runtime.h>

#include "dynb_internal.h"

namespace dynb {
namespace {

typedef __bf16 bf16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__device__ inline void locate_padded(const Segs& s, int prow, int& k, int& r) {
  k = 0;
  while (k + 1 < s.K && prow >= s.poff[k + 1]) ++k;
  r = prow - s.poff[k];
}

// out[(kh*3 + kw)*C + c][p] = in[(n, ho*stride + kh - 1, wo*stride + kw - 1)][c] for the output
// pixel (n, ho, wo) that sits at padded position p (pixel-level segments `s`), zero for
// padding positions and out-of-range taps.  One thread writes 8 consecutive positions.
__global__ __launch_bounds__(256) void im2col_t_kernel(const bf16* __restrict__ in, int64_t ldi,
                                                       int C, int H, int W, int Ho, int Wo,
                                                       int stride, bf16* __restrict__ out,
                                                       int64_t ldo, Segs s) {
  const int P = s.poff[s.K];
  const int pg = blockIdx.x * 256 + threadIdx.x;   // granule of 8 padded positions
  const int row = blockIdx.y;                      // (kh*3 + kw)*C + c
  if (pg * 8 >= P) return;
  const int tap = row / C, c = row - tap * C;
  const int kh = tap / 3, kw = tap - kh * 3;
  bf16x8 v;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int p = pg * 8 + e;
    float val = 0.f;
    int k, r;
    locate_padded(s, p, k, r);
    if (r < s.off[k + 1] - s.off[k]) {
      const int m = s.off[k] + r;                  // dense output pixel
      const int n = m / (Ho * Wo), rem = m - n * (Ho * Wo);
      const int ho = rem / Wo, wo = rem - ho * Wo;
      const int y = ho * stride + kh - 1, x = wo * stride + kw - 1;
      if (y >= 0 && y < H && x >= 0 && x < W)
        val = (float)in[((int64_t)(n * H + y) * W + x) * ldi + c];
    }
    v[e] = (bf16)val;
  }
  *(bf16x8*)(out + (int64_t)row * ldo + pg * 8) = v;
}

// pooled[n][c] = mean over the HW pixels of act[(n, pixel)][c]   (fp32 sum, bf16 store)
__global__ __launch_bounds__(256) void gap_forward_kernel(const bf16* __restrict__ act, int64_t lda,
                                                          int HW, int C, int samples,
                                                          bf16* __restrict__ pooled, int64_t ldp) {
  const int c = blockIdx.x * 256 + threadIdx.x, n = blockIdx.y;
  if (c >= C || n >= samples) return;
  float acc = 0.f;
  for (int px = 0; px < HW; ++px) acc += (float)act[((int64_t)n * HW + px) * lda + c];
  pooled[(int64_t)n * ldp + c] = (bf16)(acc / (float)HW);
}

// d act[(n, pixel)][c] = d pooled[n][c] / HW, masked by act > 0 when the pooled layer's producer
// applied a ReLU
__global__ __launch_bounds__(256) void gap_backward_kernel(const bf16* __restrict__ dpooled,
                                                           int64_t ldp, const bf16* __restrict__ act,
                                                           int64_t lda, int HW, int C, int samples,
                                                           int relu, bf16* __restrict__ dact,
                                                           int64_t ldd) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  const int64_t row = blockIdx.y;   // (n, pixel)
  if (c >= C || row >= (int64_t)samples * HW) return;
  float v = (float)dpooled[(row / HW) * ldp + c] / (float)HW;
  if (relu && !((float)act[row * lda + c] > 0.f)) v = 0.f;
  dact[row * ldd + c] = (bf16)v;
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

int launch_im2col_t(const void* in, int64_t ldi, int C, int H, int W, int Ho, int Wo, int stride,
                    void* out, int64_t ldo, const Segs& s, void* stream) {
  const int P = s.poff[s.K];
  if (P == 0) return DYNB_OK;
  Timed t(KC_CONV_AUX, stream, 0, 2.0 * 9 * C * (double)s.off[s.K] * 2);
  dim3 grid((P / 8 + 255) / 256, 9 * C);
  hipLaunchKernelGGL(im2col_t_kernel, grid, dim3(256), 0, (hipStream_t)stream, (const bf16*)in, ldi,
                     C, H, W, Ho, Wo, stride, (bf16*)out, ldo, s);
  return ok("im2col_t");
}

int launch_gap_forward(const void* act, int64_t lda, int HW, int C, int samples, void* pooled,
                       int64_t ldp, void* stream) {
  if (samples == 0) return DYNB_OK;
  Timed t(KC_CONV_AUX, stream, 0, (double)samples * HW * C * 2);
  dim3 grid((C + 255) / 256, samples);
  hipLaunchKernelGGL(gap_forward_kernel, grid, dim3(256), 0, (hipStream_t)stream, (const bf16*)act,
                     lda, HW, C, samples, (bf16*)pooled, ldp);
  return ok("gap_forward");
}

int launch_gap_backward(const void* dpooled, int64_t ldp, const void* act, int64_t lda, int HW,
                        int C, int samples, int relu, void* dact, int64_t ldd, void* stream) {
  if (samples == 0) return DYNB_OK;
  Timed t(KC_CONV_AUX, stream, 0, (double)samples * HW * C * 4);
  dim3 grid((C + 255) / 256, samples * HW);
  hipLaunchKernelGGL(gap_backward_kernel, grid, dim3(256), 0, (hipStream_t)stream,
                     (const bf16*)dpooled, ldp, (const bf16*)act, lda, HW, C, samples, relu,
                     (bf16*)dact, ldd);
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
