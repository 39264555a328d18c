// Small kernels around the GEMMs: input packing into the padded row space, transposes,
// softmax cross-entropy with the per-worker 1/b_k, bias gradients, loss reduction and the
// 16-bit weight copies.
#include <hip/hip_runtime.h>

#include "device_rows.h"
#include "dynb_internal.h"

namespace dynb {
namespace {

typedef __bf16 bf16;

template <typename T> __device__ inline T from_float(float v) { return (T)v; }
template <typename T> __device__ inline float to_float(T v) { return (float)v; }

// Padded row -> (worker, row inside the worker's padded segment).
__device__ inline void locate_padded(const Segs& s, int prow, int& k, int& r) {
  k = 0;
  while (k + 1 < s.K && prow >= s.poff[k + 1]) ++k;
  r = prow - s.poff[k];
}
// Dense row -> worker.
__device__ inline int worker_of(const Segs& s, int row) {
  int k = 0;
  while (k + 1 < s.K && row >= s.off[k + 1]) ++k;
  return k;
}

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ inline float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// ---- pack: fp32 rows -> rows of T ---------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void pack_rows_kernel(const float* __restrict__ x, int D,
                                                        T* __restrict__ out, int64_t ld) {
  const int row = blockIdx.y;
  const float* src = x + (int64_t)row * D;
  T* dst = out + (int64_t)row * ld;
  for (int c = blockIdx.x * 256 + threadIdx.x; c < D; c += gridDim.x * 256)
    dst[c] = from_float<T>(src[c]);
}

// the same for rows whose length is a multiple of 8 with 16-byte aligned rows on both sides:
// 8 elements per lane (two 16-byte loads, one 16- or two 16-byte stores), grid-stride over all
// granules of the matrix
template <typename T>
__global__ __launch_bounds__(256) void pack_rows_vec_kernel(const float* __restrict__ x,
                                                            int64_t rows, int D,
                                                            T* __restrict__ out, int64_t ld) {
  typedef float f4 __attribute__((ext_vector_type(4)));
  typedef T vec8T __attribute__((ext_vector_type(8)));
  const int gpr = D / 8;                       // granules per row
  const int64_t total = rows * gpr;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t r = i / gpr;
    const int c = (int)(i - r * gpr) * 8;
    const f4 a = __builtin_nontemporal_load((const f4*)(x + r * D + c));
    const f4 b = __builtin_nontemporal_load((const f4*)(x + r * D + c + 4));
    const vec8T v = {from_float<T>(a[0]), from_float<T>(a[1]), from_float<T>(a[2]), from_float<T>(a[3]),
                     from_float<T>(b[0]), from_float<T>(b[1]), from_float<T>(b[2]), from_float<T>(b[3])};
    *(vec8T*)(out + r * ld + c) = v;
  }
}

// rows of at most 8 features (an RGB pixel): one lane per row, one 16-byte store; the columns
// [D, 8) are written as zero, the rest of the padded row is never touched (it holds zeros)
__global__ __launch_bounds__(256) void pack_rows_narrow_kernel(const float* __restrict__ x,
                                                               int64_t rows, int D,
                                                               __bf16* __restrict__ out, int64_t ld) {
  typedef __bf16 vec8 __attribute__((ext_vector_type(8)));
  const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (r >= rows) return;
  vec8 v;
#pragma unroll
  for (int c = 0; c < 8; ++c) v[c] = c < D ? (__bf16)x[r * D + c] : (__bf16)0.f;
  *(vec8*)(out + r * ld) = v;
}

// ---- transpose into the padded row space: out[c][p] = in[m(p)][c], 0 where p is padding ----
// p runs over the padded positions; worker k's b_k rows sit at [poff_k, poff_k + b_k).
// A 64 x 64 tile moves through LDS; global loads and stores are 16 bytes per lane, and eight
// neighbouring lanes write one contiguous 128-byte line of an output row.
template <typename T>
__global__ __launch_bounds__(256) void transpose_kernel(const T* __restrict__ in, int64_t ldi,
                                                        int C, T* __restrict__ out, int64_t ldo,
                                                        Segs s) {
  constexpr int G = 16 / sizeof(T);          // elements per 16-byte granule
  constexpr int GC = 64 / G;                 // granules per tile row
  // row pitch of 33 (bf16) / 65 (fp32) dwords: the turned reads below walk down a column, and
  // rows that are 8 apart must not fall into the same LDS bank
  constexpr int PITCH = 64 + 4 / sizeof(T);
  __shared__ T tile[64][PITCH];
  const int p0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const int P = s.poff[s.K];
  typedef T vecT __attribute__((ext_vector_type(G)));
  for (int idx = threadIdx.x; idx < 64 * GC; idx += 256) {
    const int r = idx / GC, gc = idx % GC;
    const int pr = p0 + r;
    vecT v = {};
    if (pr < P) {
      int k, rl;
      locate_padded(s, pr, k, rl);
      if (rl < s.off[k + 1] - s.off[k])
        v = *(const vecT*)(in + (int64_t)(s.off[k] + rl) * ldi + c0 + gc * G);
    }
#pragma unroll
    for (int e = 0; e < G; ++e) tile[r][gc * G + e] = v[e];
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < 64 * GC; idx += 256) {
    const int rg = idx % GC, c = idx / GC;    // rg: granule of padded positions, c: output row
    if (c0 + c >= C) continue;
    vecT v;
#pragma unroll
    for (int e = 0; e < G; ++e) v[e] = tile[rg * G + e][c];
    *(vecT*)(out + (int64_t)(c0 + c) * ldo + p0 + rg * G) = v;
  }
}

// ---- softmax cross-entropy, one wavefront per row -----------------------------------------
// dz = (softmax(z) - onehot(y)) / b_k for the rows of worker k; zero in the pad columns.
template <typename T>
__global__ __launch_bounds__(256) void softmax_xent_kernel(const float* __restrict__ z, int64_t ldz,
                                                           const int32_t* __restrict__ y, int C,
                                                           T* __restrict__ dz, int64_t ldd,
                                                           int ld_cols, float* __restrict__ rowloss,
                                                           Segs s) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= s.off[s.K]) return;
  const int k = worker_of(s, row);
  const int bk = s.off[k + 1] - s.off[k];
  T* drow = dz + (int64_t)row * ldd;
  const float* zr = z + (int64_t)row * ldz;
  int label = y[row];
  label = label < 0 ? 0 : (label >= C ? C - 1 : label);   // keeps the read in bounds
  if (ld_cols <= 1024 && (ldz & 3) == 0 && (ldd & 3) == 0) {
    // the whole row in registers: 16-byte loads, one exponential per element
    typedef T vec4T __attribute__((ext_vector_type(4)));
    float4 v[4];
    float m = -INFINITY;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int c0 = 4 * (lane + 64 * u);
      v[u] = c0 < ld_cols ? *(const float4*)(zr + c0) : make_float4(0.f, 0.f, 0.f, 0.f);
      float* e = (float*)&v[u];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (c0 + q >= C) e[q] = -INFINITY;
        m = fmaxf(m, e[q]);
      }
    }
    m = wave_max(m);
    float sum = 0.f;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      float* e = (float*)&v[u];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        e[q] = expf(e[q] - m);          // (exp(-inf) = 0 in the pad columns)
        sum += e[q];
      }
    }
    sum = wave_sum(sum);
    const float inv = 1.f / sum, scale = 1.f / (float)bk;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int c0 = 4 * (lane + 64 * u);
      if (c0 >= ld_cols) continue;
      const float* e = (const float*)&v[u];
      vec4T o;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int c = c0 + q;
        o[q] = from_float<T>(c < C ? (e[q] * inv - (c == label ? 1.f : 0.f)) * scale : 0.f);
      }
      *(vec4T*)(drow + c0) = o;
    }
    if (lane == 0) rowloss[row] = logf(sum) - (zr[label] - m);
    return;
  }
  float m = -INFINITY;
  for (int c = lane; c < C; c += 64) m = fmaxf(m, zr[c]);
  m = wave_max(m);
  float sum = 0.f;
  for (int c = lane; c < C; c += 64) sum += expf(zr[c] - m);
  sum = wave_sum(sum);
  const float inv = 1.f / sum;
  const float scale = 1.f / (float)bk;
  for (int c = lane; c < ld_cols; c += 64) {
    float v = 0.f;
    if (c < C) v = (expf(zr[c] - m) * inv - (c == label ? 1.f : 0.f)) * scale;
    drow[c] = from_float<T>(v);
  }
  if (lane == 0) rowloss[row] = logf(sum) - (zr[label] - m);
}

// ---- bias gradient: one wavefront per (output feature, worker) --------------------------
// The worker's padded segment starts on a 16-byte boundary and its padding holds zeros, so the
// whole segment is summed with 16-byte loads.
template <typename T>
__global__ __launch_bounds__(256) void bias_grad_kernel(const T* __restrict__ dyT, int64_t ld,
                                                        int N, float* __restrict__ grads,
                                                        int64_t group_stride, Segs s) {
  constexpr int G = 16 / sizeof(T);
  typedef T vecT __attribute__((ext_vector_type(G)));
  const int lane = threadIdx.x & 63;
  const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int g = blockIdx.y;
  if (n >= N) return;
  const int granules = (s.poff[g + 1] - s.poff[g]) / G;
  const vecT* row = (const vecT*)(dyT + (int64_t)n * ld + s.poff[g]);
  float acc = 0.f;
  for (int i = lane; i < granules; i += 64) {
    const vecT v = row[i];
#pragma unroll
    for (int e = 0; e < G; ++e) acc += to_float<T>(v[e]);
  }
  acc = wave_sum(acc);
  if (lane == 0) grads[(int64_t)g * group_stride + n] = acc;
}

// ---- per-worker mean loss, zero tail of each worker's gradient vector, and (workgroups behind
// the first K) the weighted aggregate, Eq. 2, of the small tensors listed in r -- one launch
// for what used to be two tiny ones at the end of every step ---------------------------------
__global__ __launch_bounds__(64) void finalize_kernel(const float* __restrict__ rowloss,
                                                      float* __restrict__ loss,
                                                      float* __restrict__ grads, int64_t P,
                                                      int64_t P_pad, Segs s, Lambdas lam, Ranges r,
                                                      float* __restrict__ out, int range_bx) {
  const int lane = threadIdx.x;
  if ((int)blockIdx.x >= s.K) {
    const int q = blockIdx.x - s.K, ri = q / range_bx, bx = q % range_bx;
    const int64_t off = r.off[ri], n = r.len[ri];
    for (int64_t i = (int64_t)bx * 64 + lane; i < n; i += (int64_t)range_bx * 64) {
      float acc = 0.f;
      for (int k = 0; k < lam.K; ++k) acc += lam.w[k] * grads[(int64_t)k * P_pad + off + i];
      out[off + i] = acc;
    }
    return;
  }
  const int g = blockIdx.x;
  const int bk = s.off[g + 1] - s.off[g];
  // eight independent partial sums per lane: the loads of a round are in flight together
  float part[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int i = lane; i < bk; i += 512) {
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (i + 64 * u < bk) part[u] += rowloss[s.off[g] + i + 64 * u];
  }
  float acc = ((part[0] + part[1]) + (part[2] + part[3])) + ((part[4] + part[5]) + (part[6] + part[7]));
  acc = wave_sum(acc);
  if (lane == 0) loss[g] = bk > 0 ? acc / (float)bk : 0.f;
  if (grads)
    for (int64_t p = P + lane; p < P_pad; p += 64) grads[(int64_t)g * P_pad + p] = 0.f;
  // (the aggregate's padding is written here, not summed from the tails above: workgroups of
  // one launch run in no particular order)
  if (out && g == 0)
    for (int64_t p = P + lane; p < P_pad; p += 64) out[p] = 0.f;
}

// ---- read and discard (see launch_touch) -------------------------------------------------
__global__ __launch_bounds__(256) void touch_kernel(const uint4* __restrict__ p, int64_t n,
                                                    uint32_t* sink) {
  uint32_t acc = 0;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const uint4 v = p[i];
    acc |= v.x ^ v.y ^ v.z ^ v.w;
  }
  if (sink) *sink = acc;   // (sink is always null: the condition only keeps the loads alive)
}

// ---- weight copies: Wn[r][c] = T(W[r][c]),  Wt[c][r] = T(W[r][c]) ----------------------
template <typename T>
__global__ __launch_bounds__(256) void weight_cast_kernel(const float* __restrict__ W, int R, int C,
                                                          T* __restrict__ Wn, int64_t ldn,
                                                          T* __restrict__ Wt, int64_t ldt) {
  __shared__ float tile[64][65];
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int i = ty; i < 64; i += 4) {
    const int r = r0 + i, c = c0 + tx;
    float v = 0.f;
    if (r < R && c < C) {
      v = W[(int64_t)r * C + c];
      Wn[(int64_t)r * ldn + c] = from_float<T>(v);
    }
    tile[i][tx] = v;
  }
  __syncthreads();
  for (int i = ty; i < 64; i += 4) {
    const int c = c0 + i, r = r0 + tx;
    if (c < C && r < R) Wt[(int64_t)c * ldt + r] = from_float<T>(tile[tx][i]);
  }
}

// ---- sum of the split weight-gradient chunks, fixed order -------------------------------
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const float* __restrict__ partial,
                                                           int split, int64_t pstride, int64_t n,
                                                           float* __restrict__ out,
                                                           int64_t group_stride) {
  const int g = blockIdx.y;
  for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < n; e += (int64_t)gridDim.x * 256) {
    float acc = 0.f;
    for (int c = 0; c < split; ++c) acc += partial[((int64_t)g * split + c) * pstride + e];
    out[(int64_t)g * group_stride + e] = acc;
  }
}

inline int ok(const char* what) {
  return hipGetLastError() == hipSuccess ? DYNB_OK : fail(DYNB_ERR_HIP, "%s: launch failed", what);
}

}  // namespace

#define DISPATCH_T(dtype, CALL)                              \
  do {                                                       \
    if ((dtype) == DYNB_BF16) { typedef bf16 T; CALL; }      \
    else { typedef float T; CALL; }                          \
  } while (0)

int launch_pack_rows(int dtype, const float* x, int rows, int D, void* out, int64_t ld,
                     void* stream) {
  if (rows == 0) return DYNB_OK;
  const int es = dtype == DYNB_BF16 ? 2 : 4;
  Timed t(KC_PACK, stream, 0, (double)rows * D * (4 + es));
  if ((D & 7) == 0 && (ld & 7) == 0 && !(((uintptr_t)x | (uintptr_t)out) & 31)) {
    int64_t blocks = ((int64_t)rows * (D / 8) + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    DISPATCH_T(dtype, hipLaunchKernelGGL(pack_rows_vec_kernel<T>, dim3((unsigned)blocks), dim3(256), 0,
                                         (hipStream_t)stream, x, (int64_t)rows, D, (T*)out, ld));
    return ok("pack_rows");
  }
  if (dtype == DYNB_BF16 && D <= 8 && (ld & 7) == 0 && !((uintptr_t)out & 15)) {
    hipLaunchKernelGGL(pack_rows_narrow_kernel, dim3((unsigned)((rows + 255) / 256)), dim3(256), 0,
                       (hipStream_t)stream, x, (int64_t)rows, D, (__bf16*)out, ld);
    return ok("pack_rows");
  }
  dim3 grid((D + 255) / 256 > 8 ? 8 : (D + 255) / 256, rows);
  DISPATCH_T(dtype, hipLaunchKernelGGL(pack_rows_kernel<T>, grid, dim3(256), 0,
                                       (hipStream_t)stream, x, D, (T*)out, ld));
  return ok("pack_rows");
}

int launch_transpose(int dtype, const void* in, int64_t ldi, int C, void* out, int64_t ldo,
                     const Segs& s, void* stream) {
  const int P = s.poff[s.K];
  if (P == 0 || C == 0) return DYNB_OK;
  const int es = dtype == DYNB_BF16 ? 2 : 4;
  Timed t(KC_TRANSPOSE, stream, 0, 2.0 * s.off[s.K] * C * es);
  dim3 grid((C + 63) / 64, (P + 63) / 64);
  DISPATCH_T(dtype, hipLaunchKernelGGL(transpose_kernel<T>, grid, dim3(256), 0,
                                       (hipStream_t)stream, (const T*)in, ldi, C, (T*)out, ldo, s));
  return ok("transpose");
}

int launch_softmax_xent(int dtype, const float* logits, int64_t ldz, const int32_t* y, int C,
                        void* dz, int64_t ldd, int ld_cols, float* rowloss, const Segs& s,
                        void* stream) {
  const int rows = s.off[s.K];
  if (rows == 0) return DYNB_OK;
  Timed t(KC_SOFTMAX, stream, 0, (double)rows * C * 6);
  DISPATCH_T(dtype, hipLaunchKernelGGL(softmax_xent_kernel<T>, dim3((rows + 3) / 4), dim3(256), 0,
                                       (hipStream_t)stream, logits, ldz, y, C, (T*)dz, ldd,
                                       ld_cols, rowloss, s));
  return ok("softmax_xent");
}

// The same from the row-major gradient dy [rows][ld] (bf16): one workgroup per (64 features,
// worker); 8 lanes cover the 128 bytes of a row, 32 row-lanes walk the worker's rows, the
// partial sums meet in a fixed order.
__global__ __launch_bounds__(256) void bias_grad_rows_kernel(const bf16* __restrict__ dy, int64_t ld,
                                                             int N, float* __restrict__ grads,
                                                             int64_t group_stride, Segs s) {
  __shared__ float red[4][64];
  const int cg = threadIdx.x & 7, rl = threadIdx.x >> 3;
  const int c0 = blockIdx.x * 64 + cg * 8, k = blockIdx.y;
  const int r0 = s.off[k], n = s.off[k + 1] - r0;
  float acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) acc[j] = 0.f;
  for (int r = rl; r < n; r += 32) {
    float v[8];
    unpack8(load8(dy + (int64_t)(r0 + r) * ld + c0), v);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] += v[j];
  }
  sum_over_rows(acc, red);
  if (rl == 0) {
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (c0 + j < N) grads[(int64_t)k * group_stride + c0 + j] = acc[j];
  }
}

int launch_bias_grad_rows(const void* dy, int64_t ld, int N, float* grads, int64_t group_stride,
                          const Segs& s, void* stream) {
  if (N == 0) return DYNB_OK;
  if (ld % 64 || ld < N) return fail(DYNB_ERR_BADARG, "bias_grad_rows: the row pitch must cover whole 64-feature blocks");
  Timed t(KC_BIAS_GRAD, stream, 0, (double)s.off[s.K] * N * 2);
  hipLaunchKernelGGL(bias_grad_rows_kernel, dim3((unsigned)(ld / 64), s.K), dim3(256), 0,
                     (hipStream_t)stream, (const bf16*)dy, ld, N, grads, group_stride, s);
  return ok("bias_grad_rows");
}

int launch_bias_grad(int dtype, const void* dyT, int64_t ld, int N, float* grads,
                     int64_t group_stride, const Segs& s, void* stream) {
  const int es = dtype == DYNB_BF16 ? 2 : 4;
  Timed t(KC_BIAS_GRAD, stream, 0, (double)s.off[s.K] * N * es);
  DISPATCH_T(dtype, hipLaunchKernelGGL(bias_grad_kernel<T>, dim3((N + 3) / 4, s.K), dim3(256), 0,
                                       (hipStream_t)stream, (const T*)dyT, ld, N, grads,
                                       group_stride, s));
  return ok("bias_grad");
}

int launch_touch(const void* p, int64_t bytes, void* stream) {
  if (bytes < 16) return DYNB_OK;
  Timed t(KC_PACK, stream, 0, (double)bytes);   // (counted with the other staging passes)
  int64_t bx = (bytes / 16 + 255) / 256;
  if (bx > 2048) bx = 2048;
  hipLaunchKernelGGL(touch_kernel, dim3((unsigned)bx), dim3(256), 0, (hipStream_t)stream,
                     (const uint4*)p, bytes / 16, (uint32_t*)nullptr);
  return ok("touch");
}

int launch_finalize(const float* rowloss, float* loss, float* grads, int64_t P, int64_t P_pad,
                    const Segs& s, const Lambdas* lam, const Ranges* small, float* out, void* stream) {
  Lambdas l;
  l.K = 0;
  Ranges r;
  r.n = 0;
  int64_t longest = 0, total = 0;
  if (out && lam && small) {
    l = *lam;
    r = *small;
    for (int i = 0; i < r.n; ++i) {
      longest = r.len[i] > longest ? r.len[i] : longest;
      total += r.len[i];
    }
  }
  int64_t bx = (longest + 63) / 64;
  if (bx > 256) bx = 256;
  if (bx < 1) bx = 1;
  const int extra = longest > 0 ? (int)bx * r.n : 0;
  Timed t(KC_FINALIZE, stream, 2.0 * l.K * total, 4.0 * (l.K + 1) * total);
  hipLaunchKernelGGL(finalize_kernel, dim3(s.K + extra), dim3(64), 0, (hipStream_t)stream, rowloss, loss,
                     grads, P, P_pad, s, l, r, out, (int)bx);
  return ok("finalize");
}

int launch_wgrad_reduce(const float* partial, int split, int64_t partial_stride, int64_t n,
                        float* out, int64_t group_stride, int K, void* stream) {
  Timed t(KC_GEMM_WGRAD, stream, 0, 0);
  int64_t bx = (n + 255) / 256;
  if (bx > 1024) bx = 1024;
  hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((unsigned)bx, K), dim3(256), 0, (hipStream_t)stream,
                     partial, split, partial_stride, n, out, group_stride);
  return ok("wgrad_reduce");
}

int launch_weight_cast(int dtype, const float* W, int R, int C, void* Wn, int64_t ldn, void* Wt,
                       int64_t ldt, void* stream) {
  const int es = dtype == DYNB_BF16 ? 2 : 4;
  Timed t(KC_WEIGHT_CAST, stream, 0, (double)R * C * (4 + 2 * es));
  dim3 grid((C + 63) / 64, (R + 63) / 64);
  DISPATCH_T(dtype, hipLaunchKernelGGL(weight_cast_kernel<T>, grid, dim3(256), 0,
                                       (hipStream_t)stream, W, R, C, (T*)Wn, ldn, (T*)Wt, ldt));
  return ok("weight_cast");
}

}  // namespace dynb
