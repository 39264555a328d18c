// Ragged / grouped GEMMs  C'[i][j] = sum_k A[i][k] * B[j][k]  (both operands k-contiguous).
//   bf16: MFMA 32x32x16 with fp32 accumulators, tiles staged through LDS in 16-byte
//         granules with an XOR swizzle, software-pipelined global loads.
//   fp32: plain FMA tiles (parity path for the fp32 workloads).
// Batch sizes are run-time data: rows, columns and reduction depth are predicated, nothing
// is compiled per size.
#include <hip/hip_runtime.h>

#include "dynb_internal.h"

namespace dynb {
namespace {

typedef __bf16 bf16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct GroupView {
  int64_t col0;  // first reduction column of this group
  int depth;     // reduction length
  float* Cf;     // fp32 output base for this group
};

__device__ inline GroupView group_view(const GemmArgs& p, const Segs& s, int g) {
  GroupView v;
  if (p.mode == MODE_WGRAD) {
    v.col0 = s.poff[g];
    v.depth = s.poff[g + 1] - s.poff[g];
    v.Cf = p.Cf + (int64_t)g * p.group_stride;
  } else {
    v.col0 = 0;
    v.depth = p.K;
    v.Cf = p.Cf;
  }
  return v;
}

// Scalar epilogue shared by both kernels (T = storage type of C and mask).
template <typename T, int MODE>
__device__ inline void store_one(const GemmArgs& p, const GroupView& gv, int i, int j, float v) {
  if (MODE == MODE_FWD) {
    if (p.bias) v += p.bias[j];
    if (p.relu) v = fmaxf(v, 0.f);
    if (p.C) ((T*)p.C)[(int64_t)i * p.ldc + j] = (T)v;
    if (p.Cf) p.Cf[(int64_t)i * p.ldcf + j] = v;
  } else if (MODE == MODE_DGRAD) {
    if (p.mask && !((float)((const T*)p.mask)[(int64_t)i * p.ldmask + j] > 0.f)) v = 0.f;
    ((T*)p.C)[(int64_t)i * p.ldc + j] = (T)v;
  } else {
    gv.Cf[(int64_t)j * p.ldcf + i] = v;
  }
}

// ------------------------------------------------------------------------------------
// bf16 MFMA kernel
// ------------------------------------------------------------------------------------
constexpr int BK = 64;          // reduction elements per stage
constexpr int GPR = BK / 8;     // 16-byte granules per tile row

template <int BM, int BN, int WM, int WN, int MODE>
__global__ __launch_bounds__(WM * WN * 64) void gemm_bf16_kernel(GemmArgs p, Segs segs) {
  constexpr int NT = WM * WN * 64;
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  constexpr int LA = BM * GPR / NT, LB = BN * GPR / NT;
  static_assert(BM * GPR % NT == 0 && BN * GPR % NT == 0, "tile/threads mismatch");

  __shared__ uint4 sA[2][BM * GPR];
  __shared__ uint4 sB[2][BN * GPR];

  const GroupView gv = group_view(p, segs, blockIdx.z);
  const int i0 = blockIdx.x * BM, j0 = blockIdx.y * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WM, wn = wave / WM;

  const bf16* A = (const bf16*)p.A + gv.col0;
  const bf16* B = (const bf16*)p.B + gv.col0;

  uint4 ra[LA], rb[LB];
  auto gload = [&](int k0) {
#pragma unroll
    for (int u = 0; u < LA; ++u) {
      const int idx = tid + u * NT, row = idx / GPR, gr = idx % GPR;
      const int i = i0 + row, k = k0 + gr * 8;
      ra[u] = (i < p.M && k < gv.depth) ? *(const uint4*)(A + (int64_t)i * p.lda + k)
                                        : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < LB; ++u) {
      const int idx = tid + u * NT, row = idx / GPR, gr = idx % GPR;
      const int j = j0 + row, k = k0 + gr * 8;
      rb[u] = (j < p.N && k < gv.depth) ? *(const uint4*)(B + (int64_t)j * p.ldb + k)
                                        : make_uint4(0, 0, 0, 0);
    }
  };
  auto lstore = [&](int buf) {
#pragma unroll
    for (int u = 0; u < LA; ++u) {
      const int idx = tid + u * NT, row = idx / GPR, gr = idx % GPR;
      sA[buf][row * GPR + (gr ^ (row & 7))] = ra[u];
    }
#pragma unroll
    for (int u = 0; u < LB; ++u) {
      const int idx = tid + u * NT, row = idx / GPR, gr = idx % GPR;
      sB[buf][row * GPR + (gr ^ (row & 7))] = rb[u];
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  const int nk = (gv.depth + BK - 1) / BK;
  if (nk > 0) {
    gload(0);
    lstore(0);
  }
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) gload((kt + 1) * BK);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 fa[TM], fb[TN];
      const int gr = kk * 2 + (lane >> 5);
#pragma unroll
      for (int a = 0; a < TM; ++a) {
        const int row = wm * (BM / WM) + a * 32 + (lane & 31);
        fa[a] = *(const bf16x8*)&sA[buf][row * GPR + (gr ^ (row & 7))];
      }
#pragma unroll
      for (int b = 0; b < TN; ++b) {
        const int row = wn * (BN / WN) + b * 32 + (lane & 31);
        fb[b] = *(const bf16x8*)&sB[buf][row * GPR + (gr ^ (row & 7))];
      }
#pragma unroll
      for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
    }
    if (kt + 1 < nk) lstore(buf ^ 1);
    __syncthreads();
  }

  // accumulator element v of lane l:  i = 8*(v/4) + 4*(l/32) + v%4,  j = l%32
  const bool vec_ok = MODE == MODE_WGRAD && (p.ldcf & 3) == 0 && (((uintptr_t)gv.Cf) & 15) == 0;
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b) {
      const int j = j0 + wn * (BN / WN) + b * 32 + (lane & 31);
      if (j >= p.N) continue;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int ib = i0 + wm * (BM / WM) + a * 32 + 8 * q + 4 * (lane >> 5);
        if (MODE == MODE_WGRAD && vec_ok && ib + 3 < p.M) {
          float4 o = make_float4(acc[a][b][4 * q], acc[a][b][4 * q + 1], acc[a][b][4 * q + 2],
                                 acc[a][b][4 * q + 3]);
          *(float4*)&gv.Cf[(int64_t)j * p.ldcf + ib] = o;
        } else {
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (ib + r < p.M) store_one<bf16, MODE>(p, gv, ib + r, j, acc[a][b][4 * q + r]);
        }
      }
    }
}

// ------------------------------------------------------------------------------------
// fp32 FMA kernel: 64x64 tile, 16-deep stages, 4x4 outputs per thread
// ------------------------------------------------------------------------------------
template <int MODE>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmArgs p, Segs segs) {
  constexpr int TB = 64, TK = 16;
  __shared__ float sA[TK][TB + 4];
  __shared__ float sB[TK][TB + 4];
  const GroupView gv = group_view(p, segs, blockIdx.z);
  const int i0 = blockIdx.x * TB, j0 = blockIdx.y * TB;
  const int tid = threadIdx.x;
  const int lrow = tid >> 2, lk = (tid & 3) * 4;     // loader: one float4 per operand
  const int ti = (tid >> 4) * 4, tj = (tid & 15) * 4;  // compute: 4x4 block
  const float* A = (const float*)p.A + gv.col0;
  const float* B = (const float*)p.B + gv.col0;

  float acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) acc[a][b] = 0.f;

  for (int k0 = 0; k0 < gv.depth; k0 += TK) {
    float4 va = make_float4(0.f, 0.f, 0.f, 0.f), vb = va;
    const int k = k0 + lk;
    if (i0 + lrow < p.M && k < gv.depth) va = *(const float4*)(A + (int64_t)(i0 + lrow) * p.lda + k);
    if (j0 + lrow < p.N && k < gv.depth) vb = *(const float4*)(B + (int64_t)(j0 + lrow) * p.ldb + k);
    __syncthreads();
    sA[lk + 0][lrow] = va.x; sA[lk + 1][lrow] = va.y; sA[lk + 2][lrow] = va.z; sA[lk + 3][lrow] = va.w;
    sB[lk + 0][lrow] = vb.x; sB[lk + 1][lrow] = vb.y; sB[lk + 2][lrow] = vb.z; sB[lk + 3][lrow] = vb.w;
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < TK; ++kk) {
      const float4 a4 = *(const float4*)&sA[kk][ti];
      const float4 b4 = *(const float4*)&sB[kk][tj];
      const float av[4] = {a4.x, a4.y, a4.z, a4.w};
      const float bv[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] += av[a] * bv[b];
    }
  }
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      const int i = i0 + ti + a, j = j0 + tj + b;
      if (i < p.M && j < p.N) store_one<float, MODE>(p, gv, i, j, acc[a][b]);
    }
}

template <int BM, int BN, int WM, int WN>
void launch_bf16(const GemmArgs& a, const Segs& s, int groups, hipStream_t st) {
  dim3 grid((a.M + BM - 1) / BM, (a.N + BN - 1) / BN, groups), block(WM * WN * 64);
  switch (a.mode) {
    case MODE_FWD:
      hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, MODE_FWD>), grid, block, 0, st, a, s);
      break;
    case MODE_DGRAD:
      hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, MODE_DGRAD>), grid, block, 0, st, a, s);
      break;
    default:
      hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, MODE_WGRAD>), grid, block, 0, st, a, s);
  }
}

void launch_f32(const GemmArgs& a, const Segs& s, int groups, hipStream_t st) {
  dim3 grid((a.M + 63) / 64, (a.N + 63) / 64, groups), block(256);
  switch (a.mode) {
    case MODE_FWD:
      hipLaunchKernelGGL(gemm_f32_kernel<MODE_FWD>, grid, block, 0, st, a, s);
      break;
    case MODE_DGRAD:
      hipLaunchKernelGGL(gemm_f32_kernel<MODE_DGRAD>, grid, block, 0, st, a, s);
      break;
    default:
      hipLaunchKernelGGL(gemm_f32_kernel<MODE_WGRAD>, grid, block, 0, st, a, s);
  }
}

}  // namespace

int launch_gemm(int dtype, const GemmArgs& a, const Segs& s, void* stream) {
  if (a.M <= 0 || a.N <= 0) return DYNB_OK;
  const int es = dtype == DYNB_BF16 ? 2 : 4;
  const int gran = 16 / es;
  if ((a.lda % gran) || (a.ldb % gran) || ((uintptr_t)a.A & 15) || ((uintptr_t)a.B & 15))
    return fail(DYNB_ERR_BADARG, "gemm: operands must have 16-byte aligned rows");
  const int groups = a.mode == MODE_WGRAD ? s.K : 1;
  // algorithmic work: true (unpadded) rows only
  double flops, bytes;
  const double rows = s.off[s.K];
  if (a.mode == MODE_WGRAD) {
    flops = 2.0 * rows * a.M * a.N;
    bytes = (double)groups * a.M * a.N * 4 + rows * (a.M + a.N) * es;
  } else {
    flops = 2.0 * rows * a.N * a.K;
    bytes = rows * (a.K + a.N) * es + (double)a.N * a.K * es;
  }
  const KClass cls = a.mode == MODE_FWD ? KC_GEMM_FWD : a.mode == MODE_DGRAD ? KC_GEMM_DGRAD
                                                                              : KC_GEMM_WGRAD;
  Timed t(cls, stream, flops, bytes);
  if (dtype == DYNB_BF16)
    launch_bf16<128, 128, 2, 2>(a, s, groups, (hipStream_t)stream);
  else
    launch_f32(a, s, groups, (hipStream_t)stream);
  return hipGetLastError() == hipSuccess ? DYNB_OK : fail(DYNB_ERR_HIP, "gemm launch failed");
}

}  // namespace dynb
