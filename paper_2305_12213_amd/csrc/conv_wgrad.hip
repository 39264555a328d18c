// Per-worker weight gradient of a 3x3 convolution (NHWC, zero padding 1, stride 1 or 2; bf16),
// straight from the row-major activations:
//   dW_k[kh][kw][ci][co] = sum over worker k's output pixels p of in[src(p, kh, kw)][ci] * dy[p][co]
// The reduction runs over pixels, which are the *rows* of both operands, while an MFMA operand
// wants 8 consecutive reduction indices per lane.  Instead of building transposed copies in
// memory (a patch matrix nine times the activation), tiles are staged in LDS as they lie in
// memory ([pixel][channel]) and fetched with the LDS transpose read of gfx950
// (ds_read_b64_tr_b16): within 16 lanes, lane r supplies the address of 4 channels of pixel
// r/4, and lane l receives channel l of 4 consecutive pixels.
//
// Work split: the rows of a worker are cut into chunks of `chunk_rows` pixels; one workgroup
// takes one chunk, 64 input and 64 output channels, and all nine taps (4 waves: each owns a
// 32 x 32 corner of the 64 x 64 tile for the nine taps, 144 accumulator registers).  A stage is
// 32 pixels x one kernel row (3 taps): 3 x 4 KB of shifted input rows and 4 KB of dy, copied
// global -> LDS asynchronously into a ring of 4 stage buffers.  Chunk results go to a scratch
// area in register order and a second kernel adds the chunks of each worker in a fixed order
// (deterministic, no atomics).  The bias gradient (column sums of dy) rides along as a tenth
// "tap" whose input operand is all ones.
#include <hip/hip_runtime.h>

#include <climits>
#include <mutex>

#include "dynb_internal.h"
#include "lds_async.h"

namespace dynb {
namespace {

typedef __bf16 bf16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int S = 4;                         // stage buffers
constexpr int TILE_BYTES = 32 * 128;         // 32 pixels x 64 channels
constexpr int STAGE_BYTES = 4 * TILE_BYTES;  // three shifted input tiles + the dy tile
constexpr int PER = 4;                       // copies per wave and stage
constexpr int SLOTS = 10;                    // nine taps and the column sums of dy
constexpr int TILE_FLOATS = 4 * SLOTS * 16 * 64;   // one chunk result per 64 x 64 channel block:
                                                   // [wave][slot][16 accumulator elements][lane]

__device__ uint4 g_zeros[1];                 // what lanes outside the image or the chunk fetch

__device__ inline void wait_copies(int stages) {   // at most `stages` stages of this wave pending
  switch (stages) {
    case 0: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
    case 1: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PER) : "memory"); break;
    default: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * PER) : "memory"); break;
  }
}

__device__ inline s16x4 read_tr(uint32_t lds_addr) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (__attribute__((address_space(3))) s16x4*)(uintptr_t)lds_addr);
}

// worker, first row and row count of a chunk
__device__ inline void chunk_span(const Segs& s, const RowChunks& ch, int chunk, int& k, int& r0, int& n) {
  k = 0;
  while (k + 1 < s.K && chunk >= ch.first[k + 1]) ++k;
  r0 = s.off[k] + (chunk - ch.first[k]) * ch.rows;
  n = min(ch.rows, s.off[k + 1] - r0);
}

struct ConvWgradArgs {
  const bf16* in; int ldi;           // [samples * H * W][ldi]
  const bf16* dy; int ldd;           // [samples * Ho * Wo][ldd]
  int H, W, Ho, Wo, stride;
  float* partial;                    // [chunk][cin block][cout block][TILE_FLOATS]
  const void* zeros;                 // 16 bytes of zeros in device memory (address of g_zeros: a
                                     // kernel argument stays in scalar registers, the symbol's
                                     // address would be re-loaded around every copy)
};

__global__ __launch_bounds__(256) void conv_wgrad_chunk_kernel(ConvWgradArgs p, Segs segs, RowChunks ch) {
  __shared__ uint4 ring[S * STAGE_BYTES / 16];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int chunk = blockIdx.x, cib = blockIdx.y, cob = blockIdx.z;
  int k, r0, n;
  chunk_span(segs, ch, chunk, k, r0, n);
  const int n_blocks = (n + 31) / 32;            // 32-pixel blocks
  const int T = 3 * n_blocks;                    // stages

  // ---- global -> LDS: this lane always moves granule (lane & 7) of pixel 8*wave + lane/8 of
  // the block; pixel rows are 128 bytes, and the two 64-byte halves of rows 2,3,6,7,... are
  // swapped so that the transpose reads of 4 neighbouring pixels fall into distinct banks.
  const int prow = 8 * wave + (lane >> 3);
  const int gq = (lane & 7) ^ (((lane >> 4) & 1) << 2);     // logical granule this lane fetches
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)&ring[0];
  // output pixel of this lane in the current block: dense row, and (sample, y, x)
  int row = r0 + prow;
  int img = row / (p.Ho * p.Wo), rem = row - img * (p.Ho * p.Wo);
  int oy = rem / p.Wo, ox = rem - oy * p.Wo;
  int left = n - prow;                           // > 0 while this lane's pixel lies in the chunk
  const bf16* in_c = p.in + cib * 64 + gq * 8;
  const bf16* dy_c = p.dy + cob * 64 + gq * 8;

  auto issue = [&](int t, int kh) {              // stage t = block t/3, kernel row kh = t%3
    const uint32_t base = lds0 + (uint32_t)((t % S) * STAGE_BYTES + wave * 1024);
    // both candidate addresses are formed unconditionally (coordinates clamped into the image,
    // so always in bounds) and one is selected: no divergent branch around the copy, every
    // stage issues exactly PER copies per wave
    const bool valid = left > 0;
    const int sy = oy * p.stride + kh - 1;
    const bool row_ok = valid && sy >= 0 && sy < p.H;
    const int csy = sy < 0 ? 0 : (sy >= p.H ? p.H - 1 : sy);
    const int line = valid ? (img * p.H + csy) * p.W : 0;      // (pixel indices fit 31 bits)
#pragma unroll
    for (int kw = 0; kw < 3; ++kw) {
      const int sx = ox * p.stride + kw - 1;
      const int csx = sx < 0 ? 0 : (sx >= p.W ? p.W - 1 : sx);
      const bf16* a = in_c + (int64_t)(line + csx) * p.ldi;
      const void* src = (row_ok && sx >= 0 && sx < p.W) ? (const void*)a : p.zeros;
      async_copy_1k(src, base + kw * TILE_BYTES);
    }
    const bf16* d = dy_c + (int64_t)(valid ? row : 0) * p.ldd;
    const void* src = valid ? (const void*)d : p.zeros;
    async_copy_1k(src, base + 3 * TILE_BYTES);
  };
  auto next_block = [&]() {                      // this lane's pixel, 32 pixels on
    row += 32;
    left -= 32;
    ox += 32;
    while (ox >= p.Wo) { ox -= p.Wo; ++oy; }
    while (oy >= p.Ho) { oy -= p.Ho; ++img; }
  };

  // ---- LDS -> MFMA operands.  Wave (wci, wco) owns input channels [32*wci, +32) x output
  // channels [32*wco, +32).  Lane l: group g = l/16 reads pixels 8*(g/2) + r/4 (+4 for the
  // second half of the 8 reduction indices), channels 16*(g%2) + 4*(r%4), r = l%16.
  const int wci = wave & 1, wco = wave >> 1;
  const int g = lane >> 4, r = lane & 15;
  const int fpix = 8 * (g >> 1) + (r >> 2);
  const int fswap = (r >> 3) & 1;                // ((pixel >> 1) & 1) of every pixel this lane reads
  const uint32_t fcol = (uint32_t)((16 * (g & 1) + 4 * (r & 3)) * 2);
  const uint32_t foff_a = (uint32_t)(fpix * 128 + ((wci ^ fswap) * 64)) + fcol;
  const uint32_t foff_b = (uint32_t)(fpix * 128 + ((wco ^ fswap) * 64)) + fcol;
  auto frag = [&](uint32_t tile, uint32_t foff, int kk) {   // 8 reduction indices of k-step kk
    const uint32_t a = tile + foff + (uint32_t)(kk * 16 * 128);
    const s16x4 lo = read_tr(a), hi = read_tr(a + 4 * 128);
    const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
  };

  f32x16 acc[9], colsum;
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
#pragma unroll
  for (int v = 0; v < 16; ++v) colsum[v] = 0.f;
  // the waves of the first input-channel block that own input channels [0, 32) also sum dy over
  // the pixels: an MFMA against ones (pixels outside the chunk hold zeros in the dy tile)
  const bool sums_columns = cib == 0 && wci == 0;
  const s16x8 ones_bits = {0x3f80, 0x3f80, 0x3f80, 0x3f80, 0x3f80, 0x3f80, 0x3f80, 0x3f80};
  const bf16x8 ones = __builtin_bit_cast(bf16x8, ones_bits);

  // ---- the stage pipeline: S - 1 stages in flight, one barrier per stage ----
  int issued = 0;                                // stages issued so far (its kernel row = issued % 3)
  auto issue_next = [&]() {
    if (issued < T) {
      const int kh = issued % 3;
      issue(issued, kh);
      if (kh == 2) next_block();
      ++issued;
    }
  };
#pragma unroll
  for (int f = 0; f < S - 1; ++f) issue_next();
  for (int blk = 0; blk < n_blocks; ++blk) {
#pragma unroll
    for (int kh = 0; kh < 3; ++kh) {
      const int t = 3 * blk + kh;
      wait_copies(issued - t - 1);               // stage t of this wave has landed
      __syncthreads();                           // ... of all waves; stage t-1 is no longer read
      issue_next();                              // into the buffer of stage t-1
      const uint32_t stage = lds0 + (uint32_t)((t % S) * STAGE_BYTES);
      const bf16x8 b0 = frag(stage + 3 * TILE_BYTES, foff_b, 0);
      const bf16x8 b1 = frag(stage + 3 * TILE_BYTES, foff_b, 1);
      if (kh == 1 && sums_columns) {             // once per pixel block
        colsum = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b0, ones, colsum, 0, 0, 0);
        colsum = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b1, ones, colsum, 0, 0, 0);
      }
#pragma unroll
      for (int kw = 0; kw < 3; ++kw) {
        const bf16x8 a0 = frag(stage + kw * TILE_BYTES, foff_a, 0);
        const bf16x8 a1 = frag(stage + kw * TILE_BYTES, foff_a, 1);
        // first operand = the dimension that is contiguous in the result (output channels)
        acc[kh * 3 + kw] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b0, a0, acc[kh * 3 + kw], 0, 0, 0);
        acc[kh * 3 + kw] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b1, a1, acc[kh * 3 + kw], 0, 0, 0);
      }
    }
  }

  // ---- chunk result, in register order: [wave][slot][v/4][lane] x 4 floats ----
  float* out = p.partial + ((int64_t)(chunk * gridDim.y + cib) * gridDim.z + cob) * TILE_FLOATS;
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const f32x4 o = {acc[t][4 * q], acc[t][4 * q + 1], acc[t][4 * q + 2], acc[t][4 * q + 3]};
      *(f32x4*)&out[(((wave * SLOTS + t) * 4 + q) * 64 + lane) * 4] = o;
    }
  if (sums_columns) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const f32x4 o = {colsum[4 * q], colsum[4 * q + 1], colsum[4 * q + 2], colsum[4 * q + 3]};
      *(f32x4*)&out[(((wave * SLOTS + 9) * 4 + q) * 64 + lane) * 4] = o;
    }
  }
}

// The same for stride 1 on images exactly 32 pixels wide, where a 32-pixel block is one image
// row: a stage is one output row, and instead of nine shifted copies it stages the three
// input rows y-1, y, y+1 once, each with one pixel of (zero) border on both sides, and the three
// horizontal taps read them at a pixel offset.  5.2 KB per row and stage move into LDS instead
// of 12 KB, which is what bounds the general kernel.  Stage: 3 x 40 pixel slots (5 KB each),
// the dy row (4 KB) and 1 KB of padding = 20 copies, 5 per wave; ring of 4 stages.
constexpr int ROW_TILE = 40 * 128;               // an input row with border, 40 pixel slots
constexpr int ROW_STAGE = 3 * ROW_TILE + TILE_BYTES + 1024;
constexpr int ROW_PER = 5;                       // copies per wave and stage

__device__ inline void wait_row_copies(int stages) {
  switch (stages) {
    case 0: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
    case 1: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(ROW_PER) : "memory"); break;
    default: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * ROW_PER) : "memory"); break;
  }
}

__global__ __launch_bounds__(256) void conv_wgrad_rows_kernel(ConvWgradArgs p, Segs segs, RowChunks ch) {
  __shared__ uint4 ring[S * ROW_STAGE / 16];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int chunk = blockIdx.x, cib = blockIdx.y, cob = blockIdx.z;
  int k, r0, n;
  chunk_span(segs, ch, chunk, k, r0, n);         // r0 and n are multiples of 32: whole image rows
  const int T = n / 32;                          // stages = output rows
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)&ring[0];

  // ---- global -> LDS.  Copy c = wave + 4u (u < 5) of a stage: c < 15: input row kh = c / 5,
  // pixel slots [8o, 8o+8), o = c % 5 (slot hx holds source pixel x = hx - 1); 15 <= c < 19:
  // pixels [8(c-15), +8) of the dy row; c = 19: padding.  This lane moves slot lane/8 of the
  // eight, granule lane%8; halves of slots 2,3,6,7,... are swapped as in the kernel above.
  // Rows are contiguous in memory across images, so every copy keeps a running pointer that
  // moves on by one row per stage; whether a neighbouring row lies inside the image is the same
  // for the whole wave.  (Cycle counters showed the address arithmetic of this step, done from
  // scratch with 64-bit products, taking longer than the MFMAs of a stage.)
  const int gq = (lane & 7) ^ (((lane >> 4) & 1) << 2);
  const char* ptr[ROW_PER];                      // this lane's source in the stage's row, or nullptr
  int kind[ROW_PER];                             // 0..2: input row kh, 3: dy, 4: zeros
  const int o0 = r0 / 32;                        // first output row (image * H + y)
#pragma unroll
  for (int u = 0; u < ROW_PER; ++u) {
    const int c = wave + 4 * u;
    kind[u] = 4;
    ptr[u] = nullptr;
    if (c < 15) {
      const int x = 8 * (c % 5) + (lane >> 3) - 1;
      if (x >= 0 && x < 32) {
        kind[u] = c / 5;
        ptr[u] = (const char*)(p.in + ((int64_t)(o0 + c / 5 - 1) * 32 + x) * p.ldi + cib * 64 + gq * 8);
      }
    } else if (c < 19) {
      kind[u] = 3;
      ptr[u] = (const char*)(p.dy + ((int64_t)o0 * 32 + 8 * (c - 15) + (lane >> 3)) * p.ldd + cob * 64 + gq * 8);
    }
  }
  const int64_t in_step = (int64_t)32 * p.ldi * 2, dy_step = (int64_t)32 * p.ldd * 2;   // bytes per row
  int iy = o0 % p.H;                             // image row of the next stage to issue
  auto issue = [&](int t) {
    const uint32_t base = lds0 + (uint32_t)((t % S) * ROW_STAGE);
    const bool above = iy > 0, below = iy < p.H - 1;   // rows y-1 / y+1 exist
#pragma unroll
    for (int u = 0; u < ROW_PER; ++u) {
      const int c = wave + 4 * u;
      const bool row_ok = kind[u] == 0 ? above : (kind[u] == 2 ? below : true);
      const void* src = (ptr[u] != nullptr && row_ok) ? (const void*)ptr[u] : p.zeros;
      const uint32_t dst = c < 15 ? (uint32_t)((c / 5) * ROW_TILE + (c % 5) * 1024)
                                  : (uint32_t)(3 * ROW_TILE + (c - 15) * 1024);
      async_copy_1k(src, base + dst);
      if (ptr[u] != nullptr) ptr[u] += kind[u] == 3 ? dy_step : in_step;
    }
    if (++iy == p.H) iy = 0;
  };

  // ---- LDS -> MFMA operands (see the kernel above); input rows are read at slot x + kw
  const int wci = wave & 1, wco = wave >> 1;
  const int g = lane >> 4, r = lane & 15;
  const uint32_t fcol = (uint32_t)((16 * (g & 1) + 4 * (r & 3)) * 2);
  uint32_t foff_a[3];
#pragma unroll
  for (int kw = 0; kw < 3; ++kw) {
    const int hx = 8 * (g >> 1) + (r >> 2) + kw;
    foff_a[kw] = (uint32_t)(hx * 128 + ((wci ^ ((hx >> 1) & 1)) * 64)) + fcol;
  }
  const int fpix = 8 * (g >> 1) + (r >> 2);
  const uint32_t foff_b = (uint32_t)(fpix * 128 + ((wco ^ ((r >> 3) & 1)) * 64)) + fcol;
  auto frag = [&](uint32_t tile, uint32_t foff, int kk) {
    const uint32_t a = tile + foff + (uint32_t)(kk * 16 * 128);
    const s16x4 lo = read_tr(a), hi = read_tr(a + 4 * 128);
    const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
  };

  f32x16 acc[9], colsum;
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
#pragma unroll
  for (int v = 0; v < 16; ++v) colsum[v] = 0.f;
  const bool sums_columns = cib == 0 && wci == 0;
  const s16x8 ones_bits = {0x3f80, 0x3f80, 0x3f80, 0x3f80, 0x3f80, 0x3f80, 0x3f80, 0x3f80};
  const bf16x8 ones = __builtin_bit_cast(bf16x8, ones_bits);

  int issued = 0;
#pragma unroll
  for (int f = 0; f < S - 1; ++f)
    if (issued < T) { issue(issued); ++issued; }
  for (int t = 0; t < T; ++t) {
    wait_row_copies(issued - t - 1);             // stage t of this wave has landed
    __syncthreads();                             // ... of all waves; stage t-1 is no longer read
    if (issued < T) { issue(issued); ++issued; }
    const uint32_t stage = lds0 + (uint32_t)((t % S) * ROW_STAGE);
    const bf16x8 b0 = frag(stage + 3 * ROW_TILE, foff_b, 0);
    const bf16x8 b1 = frag(stage + 3 * ROW_TILE, foff_b, 1);
    // the operands of tap n+1 are fetched before the MFMAs of tap n (two register sets), so
    // that the LDS latency hides behind them; the column sums run in every wave (no branch in
    // the loop), only the waves that own them write them out
    bf16x8 a0[2], a1[2];
    a0[0] = frag(stage, foff_a[0], 0);
    a1[0] = frag(stage, foff_a[0], 1);
#pragma unroll
    for (int tap = 0; tap < 9; ++tap) {
      if (tap + 1 < 9) {
        const int nh = (tap + 1) / 3, nw = (tap + 1) - 3 * nh;
        a0[(tap + 1) & 1] = frag(stage + nh * ROW_TILE, foff_a[nw], 0);
        a1[(tap + 1) & 1] = frag(stage + nh * ROW_TILE, foff_a[nw], 1);
      }
      __builtin_amdgcn_sched_barrier(0);         // (keeps the fetches in front of the MFMAs)
      if (tap == 4) {
        colsum = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b0, ones, colsum, 0, 0, 0);
        colsum = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b1, ones, colsum, 0, 0, 0);
      }
      acc[tap] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b0, a0[tap & 1], acc[tap], 0, 0, 0);
      acc[tap] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b1, a1[tap & 1], acc[tap], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  float* out = p.partial + ((int64_t)(chunk * gridDim.y + cib) * gridDim.z + cob) * TILE_FLOATS;
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const f32x4 o = {acc[t][4 * q], acc[t][4 * q + 1], acc[t][4 * q + 2], acc[t][4 * q + 3]};
      *(f32x4*)&out[(((wave * SLOTS + t) * 4 + q) * 64 + lane) * 4] = o;
    }
  if (sums_columns) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const f32x4 o = {colsum[4 * q], colsum[4 * q + 1], colsum[4 * q + 2], colsum[4 * q + 3]};
      *(f32x4*)&out[(((wave * SLOTS + 9) * 4 + q) * 64 + lane) * 4] = o;
    }
  }
}

// dW_k[tap][ci][co .. co+3] = the chunk results of worker k added in a fixed order; the items
// behind the weights are the bias gradients db_k[co .. co+3] (slot 9, input channel 0).
// 256 threads = 32 items x 8 chunk-lanes: lane q adds chunks q, q+8, ... (four independent
// partial sums, so that the loads overlap), then the lanes are added in ascending order.
// Neighbouring threads take neighbouring input channels, which lie 16 bytes apart in a chunk
// result.  Accumulator element v of lane l belongs to output channel 8*(v/4) + 4*(l/32) + v%4
// and input channel l%32 of the wave's corner.
__global__ __launch_bounds__(256) void conv_wgrad_reduce_kernel(const float* __restrict__ partial,
                                                                int Cin, int Cout, int cibs, int cobs,
                                                                float* __restrict__ dW,
                                                                float* __restrict__ db,
                                                                int64_t group_stride, RowChunks ch) {
  __shared__ f32x4 red[8][32];
  const int il = threadIdx.x & 31, q = threadIdx.x >> 5;
  const int k = blockIdx.y;
  const int quads = (Cout + 3) / 4;
  const int64_t n_weight = (int64_t)9 * quads * Cin;
  int64_t idx = (int64_t)blockIdx.x * 32 + il;   // ((tap, quad of co), ci) | quad
  const bool live = idx < n_weight + quads;
  if (!live) idx = 0;
  const bool bias = idx >= n_weight;
  const int ci = bias ? 0 : (int)(idx % Cin);
  const int64_t tq = bias ? 0 : idx / Cin;
  const int quad = bias ? (int)(idx - n_weight) : (int)(tq % quads);
  const int slot = bias ? 9 : (int)(tq / quads);
  const int co = quad * 4;
  const int cib = ci >> 6, cob = co >> 6, cil = ci & 63, col = co & 63;
  const int wave = (cil >> 5) + 2 * (col >> 5);
  const int c32 = col & 31;
  const int lane = (cil & 31) + 32 * ((c32 & 7) >> 2);
  const int64_t within = ((int64_t)((wave * SLOTS + slot) * 4 + (c32 >> 3)) * 64 + lane) * 4;
  const int64_t stride = (int64_t)cibs * cobs * TILE_FLOATS;
  const float* src = partial + ((int64_t)cib * cobs + cob) * TILE_FLOATS + within;
  const int last = ch.first[k + 1];
  f32x4 a0 = {0.f, 0.f, 0.f, 0.f}, a1 = a0, a2 = a0, a3 = a0;
  int c = ch.first[k] + q;
  for (; c + 24 < last; c += 32) {
    a0 += *(const f32x4*)(src + c * stride);
    a1 += *(const f32x4*)(src + (c + 8) * stride);
    a2 += *(const f32x4*)(src + (c + 16) * stride);
    a3 += *(const f32x4*)(src + (c + 24) * stride);
  }
  for (; c < last; c += 8) a0 += *(const f32x4*)(src + c * stride);
  red[q][il] = (a0 + a1) + (a2 + a3);
  __syncthreads();
  if (q != 0 || !live) return;
  f32x4 sum = red[0][il];
#pragma unroll
  for (int i = 1; i < 8; ++i) sum += red[i][il];
  float* dst = bias ? db + (int64_t)k * group_stride + co
                    : dW + (int64_t)k * group_stride + ((int64_t)slot * Cin + ci) * Cout + co;
#pragma unroll
  for (int e = 0; e < 4; ++e)
    if (co + e < Cout) dst[e] = sum[e];
}

}  // namespace

// address of g_zeros on the current device (looked up once per device)
const void* device_zero_granule() {
  static std::mutex mu;
  static const void* known[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  std::lock_guard<std::mutex> lk(mu);
  if (!known[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_zeros)) != hipSuccess) return nullptr;
    known[dev] = p;
  }
  return known[dev];
}

RowChunks make_row_chunks(const Segs& s, int rows) {
  RowChunks ch;
  ch.rows = rows;
  ch.first[0] = 0;
  for (int k = 0; k < s.K; ++k)
    ch.first[k + 1] = ch.first[k] + (s.off[k + 1] - s.off[k] + rows - 1) / rows;
  for (int k = s.K + 1; k <= DYNB_MAX_WORKERS; ++k) ch.first[k] = ch.first[s.K];
  return ch;
}

int conv_wgrad_chunk_rows(int64_t max_rows) {
  // about two chunks per compute unit at the largest batch, whole 32-pixel blocks, and long
  // enough that a chunk's result (147 KB per channel block) is small against what it reads
  int64_t rows = round_up((max_rows + 511) / 512, 32);
  return (int)(rows < 256 ? 256 : rows);
}

int64_t conv_wgrad_scratch_floats(int64_t max_rows, int max_workers, int Cin, int Cout) {
  const int64_t chunks = (max_rows + conv_wgrad_chunk_rows(max_rows) - 1) / conv_wgrad_chunk_rows(max_rows) +
                         max_workers;
  return chunks * ((Cin + 63) / 64) * ((Cout + 63) / 64) * TILE_FLOATS;
}

int launch_conv_wgrad(const void* in, int64_t ldi, int Cin, int H, int W, const void* dy, int64_t ldd,
                      int Cout, int Ho, int Wo, int stride, int chunk_rows, float* scratch,
                      int64_t scratch_floats, float* dW, float* db, int64_t group_stride,
                      const Segs& s, double flops, double bytes, void* stream) {
  if (Cin <= 0 || Cout <= 0) return DYNB_OK;
  const int cibs = (Cin + 63) / 64, cobs = (Cout + 63) / 64;
  if (ldi % 64 || ldd % 64 || ldi < 64 * cibs || ldd < 64 * cobs || chunk_rows < 32 || chunk_rows % 32 ||
      (((uintptr_t)in | (uintptr_t)dy | (uintptr_t)scratch) & 15))
    return fail(DYNB_ERR_BADARG, "conv_wgrad: pitches must cover whole 64-channel blocks, 16-byte aligned");
  if (ldi > INT_MAX || ldd > INT_MAX || (int64_t)s.off[s.K] * stride * stride > INT_MAX / 2)
    return fail(DYNB_ERR_UNSUPPORTED, "conv_wgrad: tensor too large for 32-bit pixel indices");
  const void* zeros = device_zero_granule();
  if (!zeros) return fail(DYNB_ERR_HIP, "conv_wgrad: no address for the zero granule");
  const RowChunks ch = make_row_chunks(s, chunk_rows);
  const int nch = ch.first[s.K];
  if ((int64_t)nch * cibs * cobs * TILE_FLOATS > scratch_floats)
    return fail(DYNB_ERR_BADARG, "conv_wgrad: scratch area too small");
  Timed t(KC_GEMM_WGRAD, stream, flops, bytes);
  if (nch > 0) {
    ConvWgradArgs a = {(const bf16*)in, (int)ldi, (const bf16*)dy, (int)ldd, H, W, Ho, Wo, stride,
                       scratch, zeros};
    // whole image rows per chunk and per worker: the row-staged kernel applies
    bool by_rows = stride == 1 && W == 32 && Wo == 32 && H == Ho && chunk_rows % 32 == 0;
    for (int k = 0; k <= s.K && by_rows; ++k) by_rows = s.off[k] % 32 == 0;
    if (by_rows)
      hipLaunchKernelGGL(conv_wgrad_rows_kernel, dim3(nch, cibs, cobs), dim3(256), 0,
                         (hipStream_t)stream, a, s, ch);
    else
      hipLaunchKernelGGL(conv_wgrad_chunk_kernel, dim3(nch, cibs, cobs), dim3(256), 0,
                         (hipStream_t)stream, a, s, ch);
  }
  const int64_t items = (int64_t)(9 * Cin + 1) * ((Cout + 3) / 4);
  hipLaunchKernelGGL(conv_wgrad_reduce_kernel, dim3((unsigned)((items + 31) / 32), s.K), dim3(256), 0,
                     (hipStream_t)stream, scratch, Cin, Cout, cibs, cobs, dW, db, group_stride, ch);
  return hipGetLastError() == hipSuccess ? DYNB_OK : fail(DYNB_ERR_HIP, "conv_wgrad: launch failed");
}

}  // namespace dynb
