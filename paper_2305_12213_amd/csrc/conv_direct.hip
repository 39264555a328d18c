// 3x3 convolution, stride 1, zero padding 1, on images 32 pixels wide (bf16 NHWC): forward
// and input gradient as an implicit GEMM whose A operand is read from ONE halo tile in LDS.
//
// The gathered-operand GEMM fetches, for every tap, its own shifted copy of the tile's input
// rows (9 x 32 KB per 256 pixels and 64 channels) and is bound by the rate at which a compute
// unit can pull data into LDS.  Here a workgroup takes 8 image rows (256 output pixels) x 64
// output channels, copies the 10 x 34 pixels those rows and their neighbours cover into LDS
// once per 64 input channels (43 KB, zeros outside the image), and every tap reads its MFMA
// operand from that tile at a pixel offset.  Only the weights are streamed per tap (8 KB).
//
// LDS rows are 128 bytes (64 channels of a pixel, or of a weight row); the 16-byte granule g of
// row r sits at slot g ^ slot_swizzle(r).  A 16-byte operand read serves 16 lanes = 16
// neighbouring rows per clock (64 banks of 4 bytes, two rows per pass over the banks): the
// eight rows of equal parity among them need eight different swizzles.  Copies are asynchronous (global -> LDS without registers), completion is
// tracked with vmcnt by hand, as in gemm.hip.
#include <hip/hip_runtime.h>

#include "dynb_internal.h"
#include "lds_async.h"

namespace dynb {
namespace {

typedef __bf16 bf16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int HALO_W = 34, HALO_H = 10, HALO_PIX = HALO_W * HALO_H;   // 340 pixels
constexpr int HALO_COPIES = 44;             // 1 KB each (8 pixels): 11 per wave, 352 pixel slots
constexpr int WSTAGES = 3;                  // ring of weight stages (one tap x 64 channels: 8 KB)
constexpr int EP = 64 + 4;                  // epilogue patch row pitch in floats

// bits 1..3 of the row, rotated (rows r and r+8 differ in the lowest bit, rows 2 apart in the
// upper two: also conflict-free if lanes l and l+32, which read granules g and g^1, are paired)
__device__ inline int slot_swizzle(int r) { return (((r >> 1) & 3) << 1) | ((r >> 3) & 1); }

struct ConvDirectArgs {
  const bf16* src; int lds;          // [images * H * 32][lds]
  const bf16* w; int ldw;            // [N][9 * cp]: w[j][tap * cp + c]
  int H, cp, N;                      // image height (a multiple of 8), channels per tap (x64)
  int flip;                          // 0: tap (kh, kw) reads pixel (y + kh - 1, x + kw - 1);
                                     // 1: (y + 1 - kh, x + 1 - kw)  (input gradient)
  const float* bias; int relu;       // forward
  bf16* out; int64_t ldo;            // [images * H * 32][ldo]
  const bf16* mask; int64_t ldmask;  // input gradient: zero where mask <= 0 (optional)
  const bf16* addend; int64_t ldadd; // input gradient: added after rounding (optional)
  const void* zeros;                 // 16 bytes of zeros in device memory
};

__global__ __launch_bounds__(256, 2) void conv_direct_kernel(ConvDirectArgs p) {
  __shared__ uint4 halo[HALO_COPIES * 64];
  __shared__ uint4 wring[WSTAGES][512];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int tiles_per_image = p.H / 8;
  const int img = blockIdx.x / tiles_per_image, y0 = (blockIdx.x - img * tiles_per_image) * 8;
  const int j0 = blockIdx.y * 64;
  const int nblk = p.cp / 64, total = nblk * 9;
  const uint32_t lds_halo = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)&halo[0];
  const uint32_t lds_w = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)&wring[0][0];

  // ---- copy plans.  Halo copy c = wave + 4u moves halo pixels [8c, 8c+8): this lane pixel
  // 8c + lane/8, LDS slot lane%8, i.e. logical granule (lane%8) ^ slot_swizzle(pixel).
  uint32_t hoff[11];                 // byte offset of the lane's granule in src, ~0u: zeros
#pragma unroll
  for (int u = 0; u < 11; ++u) {
    const int pi = (wave + 4 * u) * 8 + (lane >> 3);
    const int hr = pi / HALO_W, hx = pi - hr * HALO_W;
    const int sy = y0 + hr - 1, sx = hx - 1;
    const int lg = (lane & 7) ^ slot_swizzle(pi);
    const bool ok = pi < HALO_PIX && sy >= 0 && sy < p.H && sx >= 0 && sx < 32;
    hoff[u] = ok ? (uint32_t)((((img * p.H + sy) * 32 + sx) * p.lds + lg * 8) * 2) : ~0u;
  }
  // weight copy c = wave + 4u (u < 2) moves rows [8c, 8c+8) of the stage: row 8c + lane/8
  uint32_t woff[2];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int row = (wave + 4 * u) * 8 + (lane >> 3);
    int j = j0 + row;
    j = j < p.N ? j : p.N - 1;       // rows past the last channel repeat it (never stored)
    const int lg = (lane & 7) ^ slot_swizzle(row);
    woff[u] = (uint32_t)((j * p.ldw + lg * 8) * 2);
  }
  const char* srcb = (const char*)p.src;
  const char* wb = (const char*)p.w;
  auto issue_halo = [&](int blk) {
#pragma unroll
    for (int u = 0; u < 11; ++u) {
      const void* s = hoff[u] != ~0u ? (const void*)(srcb + hoff[u] + (uint32_t)(blk * 128)) : p.zeros;
      async_copy_1k(s, lds_halo + (uint32_t)((wave + 4 * u) * 1024));
    }
  };
  auto issue_w = [&](int s) {        // stage s = (channel block, tap)
    const int blk = s / 9, tap = s - blk * 9;
    const uint32_t kbyte = (uint32_t)((tap * p.cp + blk * 64) * 2);
#pragma unroll
    for (int u = 0; u < 2; ++u)
      async_copy_1k(wb + woff[u] + kbyte, lds_w + (uint32_t)((s % WSTAGES) * 8192 + (wave + 4 * u) * 1024));
  };

  // ---- operand reads.  Wave w owns image rows 2w, 2w+1 of the tile (64 pixels) x 64 channels.
  // A: lane reads pixel (row, x = lane%32) shifted by the tap, granule 2kk + lane/32.
  // B: lane reads weight row b*32 + lane%32.
  const int x = lane & 31, hi = lane >> 5;
  const uint32_t brow0 = (uint32_t)(x * 128), bsw = (uint32_t)slot_swizzle(x);
  auto a_frag = [&](int a, int dy_, int dx_, int kk) {
    const int pi = (2 * wave + a + dy_) * HALO_W + x + dx_;
    const uint32_t addr = (uint32_t)(pi * 128) + (uint32_t)(((2 * kk + hi) ^ slot_swizzle(pi)) * 16);
    return *(const bf16x8*)((const char*)&halo[0] + addr);
  };
  auto b_frag = [&](int st, int b, int kk) {
    const uint32_t addr = brow0 + (uint32_t)(b * 32 * 128) + (((uint32_t)(2 * kk + hi) ^ bsw) * 16);
    return *(const bf16x8*)((const char*)&wring[st][0] + addr);
  };

  // bias of this lane's 8 output channels in the epilogue (fetched here: its latency hides
  // behind the main loop; clamped index and a select instead of a branch per channel)
  float bv[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int j = j0 + (lane & 7) * 8 + e;
    const float t = p.bias ? p.bias[j < p.N ? j : p.N - 1] : 0.f;
    bv[e] = j < p.N ? t : 0.f;
  }
  f32x16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  // ---- pipeline: the halo of a channel block, then its nine taps; weights two stages ahead.
  // Within a tap the operands of k-step kk+1 are fetched between the MFMAs of k-step kk (a wave
  // issues in order: fetches in front of the MFMAs that need them expose the LDS latency four
  // times per tap); across taps only the first k-step's fetches follow the barrier. ----
  issue_halo(0);
  issue_w(0);
  if (total > 1) issue_w(1);
  int s = 0;
  bf16x8 fa[2][2], fb[2][2];         // [register set][fragment]
  for (int blk = 0; blk < nblk; ++blk) {
#pragma unroll
    for (int tap = 0; tap < 9; ++tap, ++s) {
      // copies complete in order: all but the weights of stage s+1 (issued last) must be done;
      // at the start of a later block the halo was issued after them, so everything must be
      if (s + 1 < total && !(tap == 0 && blk > 0))
        asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
      else
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();               // stage s and the halo visible; stage s-1 no longer read
      if (s + 2 < total) issue_w(s + 2);
      const int kh = tap / 3, kw = tap - 3 * kh;
      const int dy_ = p.flip ? 2 - kh : kh, dx_ = p.flip ? 2 - kw : kw;
      const int st = s % WSTAGES;
      fa[0][0] = a_frag(0, dy_, dx_, 0); fb[0][0] = b_frag(st, 0, 0);
      fa[0][1] = a_frag(1, dy_, dx_, 0); fb[0][1] = b_frag(st, 1, 0);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const int c = kk & 1, n = c ^ 1;
        acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[c][0], fa[c][0], acc[0][0], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (kk < 3) { fa[n][0] = a_frag(0, dy_, dx_, kk + 1); fb[n][0] = b_frag(st, 0, kk + 1); }
        __builtin_amdgcn_sched_barrier(0);
        acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[c][1], fa[c][0], acc[0][1], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (kk < 3) { fa[n][1] = a_frag(1, dy_, dx_, kk + 1); fb[n][1] = b_frag(st, 1, kk + 1); }
        __builtin_amdgcn_sched_barrier(0);
        acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[c][0], fa[c][1], acc[1][0], 0, 0, 0);
        acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[c][1], fa[c][1], acc[1][1], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    __syncthreads();                 // every wave is done with this block's halo
    if (blk + 1 < nblk) issue_halo(blk + 1);
  }

  // ---- epilogue: each wave passes its 64 x 64 strip, 32 pixels at a time, through an fp32
  // patch in the (now free) halo area: 4 consecutive channels per lane become 8, and bias /
  // ReLU / addend / mask, the bf16 conversion and the stores run on whole 128-byte rows.
  float* patch = (float*)&halo[0] + wave * 32 * EP;
  // the mask and addend rows of the whole strip are fetched up front (one round trip to
  // memory instead of eight)
  const int hi4 = 4 * hi;
  const int rrow = lane >> 3, rcol = (lane & 7) * 8;
  const int jcol = j0 + rcol;
  const bool col_ok = jcol + 7 < p.N;
  const int64_t row0 = (int64_t)(img * p.H + y0 + 2 * wave) * 32;   // first pixel of the wave's strip
  bf16x8 mk[2][4], ad[2][4];
  if (col_ok) {
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int64_t i = row0 + a * 32 + rrow + 8 * t;
        if (p.mask) mk[a][t] = *(const bf16x8*)(p.mask + i * p.ldmask + jcol);
        if (p.addend) ad[a][t] = *(const bf16x8*)(p.addend + i * p.ldadd + jcol);
      }
  }

#pragma unroll
  for (int a = 0; a < 2; ++a) {
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const f32x4 o = {acc[a][b][4 * q], acc[a][b][4 * q + 1], acc[a][b][4 * q + 2], acc[a][b][4 * q + 3]};
        *(f32x4*)&patch[x * EP + b * 32 + 8 * q + hi4] = o;
      }
    __builtin_amdgcn_wave_barrier();
    f32x4 plo[4], phi[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      plo[t] = *(const f32x4*)&patch[(rrow + 8 * t) * EP + rcol];
      phi[t] = *(const f32x4*)&patch[(rrow + 8 * t) * EP + rcol + 4];
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int r = rrow + 8 * t;
      const int64_t i = row0 + a * 32 + r;
      const f32x4 lo = plo[t], hi_ = phi[t];
      if (jcol >= p.N) continue;
      float v[8] = {lo[0], lo[1], lo[2], lo[3], hi_[0], hi_[1], hi_[2], hi_[3]};
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] += bv[e];
      if (p.relu) {
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = fmaxf(v[e], 0.f);
      }
      if (col_ok) {
        if (p.addend) {
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] = (float)(bf16)v[e] + (float)ad[a][t][e];
        }
        if (p.mask) {
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (!((float)mk[a][t][e] > 0.f)) v[e] = 0.f;
        }
        const bf16x8 o = {(bf16)v[0], (bf16)v[1], (bf16)v[2], (bf16)v[3],
                          (bf16)v[4], (bf16)v[5], (bf16)v[6], (bf16)v[7]};
        *(bf16x8*)(p.out + i * p.ldo + jcol) = o;
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int j = jcol + e;
          if (j >= p.N) continue;
          float w = v[e];
          if (p.addend) w = (float)(bf16)w + (float)p.addend[i * p.ldadd + j];
          if (p.mask && !((float)p.mask[i * p.ldmask + j] > 0.f)) w = 0.f;
          p.out[i * p.ldo + j] = (bf16)w;
        }
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
}

}  // namespace

// Does the halo-tile kernel cover this convolution?  (stride 1, images 32 wide and a multiple
// of 8 high, whole 64-channel blocks per tap, tensors below 2 GiB, no fp32 output)
bool conv_direct_applies(int dtype, const GemmArgs& a) {
  if (dtype != DYNB_BF16 || !a.conv || a.mode == MODE_WGRAD || a.stride != 1) return false;
  if (a.src_w != 32 || a.row_w != 32 || a.src_h != a.row_h || a.src_h % 8 || a.cp % 64) return false;
  if (a.Cf || !a.C || a.M % (a.src_h * 32) || a.lda < a.cp || a.ldb < 9 * a.cp) return false;
  if ((int64_t)a.M * a.lda * 2 >= ((int64_t)1 << 31) || (int64_t)a.N * a.ldb * 2 >= ((int64_t)1 << 31))
    return false;
  return true;
}

int launch_conv_direct(const GemmArgs& a, void* stream) {
  const void* zeros = device_zero_granule();
  if (!zeros) return fail(DYNB_ERR_HIP, "conv_direct: no address for the zero granule");
  ConvDirectArgs p = {};
  p.src = (const bf16*)a.A; p.lds = (int)a.lda;
  p.w = (const bf16*)a.B; p.ldw = (int)a.ldb;
  p.H = a.src_h; p.cp = a.cp; p.N = a.N;
  p.flip = a.conv == 2;
  p.bias = a.mode == MODE_FWD ? a.bias : nullptr;
  p.relu = a.mode == MODE_FWD ? a.relu : 0;
  p.out = (bf16*)a.C; p.ldo = a.ldc;
  p.mask = a.mode == MODE_DGRAD ? (const bf16*)a.mask : nullptr; p.ldmask = a.ldmask;
  p.addend = a.mode == MODE_DGRAD ? (const bf16*)a.addend : nullptr; p.ldadd = a.ldadd;
  p.zeros = zeros;
  dim3 grid(a.M / 256, (a.N + 63) / 64);
  hipLaunchKernelGGL(conv_direct_kernel, grid, dim3(256), 0, (hipStream_t)stream, p);
  return hipGetLastError() == hipSuccess ? DYNB_OK : fail(DYNB_ERR_HIP, "conv_direct: launch failed");
}

}  // namespace dynb
